"""lshe_decode_step_noalloc -- the decode step with its scratch memory in the library's own
device array -- against lshe_decode_step with a caller-supplied workspace, through the C ABI.

Both run the same kernels, so every integer result (victims, scores, codes, cache contents) must
be identical and the attention outputs must agree within the attention tolerance.  The file is
collected last on purpose: it must pass on its own in a fresh process and after every other test.
"""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def H():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    from paper_2412_16187_amd import binding
    binding.lib()
    import harness
    return harness


class _Twin:
    """Two caches of one workload after the same prompt: `a` steps through lshe_decode_step,
    `b` through lshe_decode_step_noalloc."""

    def __init__(self, H, w):
        import torch
        self.H, self.w, self.torch = H, w, torch
        self.K, self.V, self.Q = H.gen_units(w)
        self.a, self.b = H.make_cache(w), H.make_cache(w)
        N = w.n_prompt
        for dc in (self.a, self.b):
            dc.prefill(H.to_device(self.K[:, :N], w.dtype), H.to_device(self.V[:, :N], w.dtype),
                       H.to_device(self.Q[:, :, :N], w.dtype), N)
        U, G = w.n_units, w.gqa_group
        dev = self.a.device
        self.dbg = [dict(scores=torch.full((U, w.budget), -9, dtype=torch.int32, device=dev),
                         codes=torch.zeros((U, G + 1, self.a.W), dtype=torch.int32, device=dev),
                         mass=torch.full((U, G), -1.0, dtype=torch.float32, device=dev))
                    for _ in range(2)]

    def inputs(self, i):
        H, w = self.H, self.w
        t = w.n_prompt + i
        pos = self.torch.full((w.batch,), t, dtype=self.torch.int32, device=self.a.device)
        return (H.to_device(self.Q[:, :, t], w.dtype), H.to_device(self.K[:, t], w.dtype),
                H.to_device(self.V[:, t], w.dtype), pos)

    def step_reference(self, i):
        q, k, v, pos = self.inputs(i)
        d = self.dbg[0]
        self.a.decode_step(q, k, v, pos, scores_dbg=d["scores"], codes_dbg=d["codes"],
                           evicted_mass=d["mass"])

    def step_noalloc(self, i):
        from paper_2412_16187_amd import binding as B
        q, k, v, pos = self.inputs(i)
        b, d = self.b, self.dbg[1]
        B.lshe_decode_step_noalloc(b.cfg, b.R_dev, q, k, v, pos, b.K, b.V, b.code, b.slot_pos,
                                   b.n_valid, b.out, b.evicted, d["scores"], d["codes"], d["mass"])

    def compare(self, what):
        torch, a, b = self.torch, self.a, self.b
        torch.cuda.synchronize()
        assert torch.equal(a.evicted, b.evicted), what
        for x, y in zip(a.snapshot(), b.snapshot()):
            assert torch.equal(x, y), what
        assert torch.equal(self.dbg[0]["scores"], self.dbg[1]["scores"]), what
        assert torch.equal(self.dbg[0]["codes"], self.dbg[1]["codes"]), what
        self.H.assert_attention_close(b.out.float().cpu().numpy(),
                                      a.out.float().cpu().numpy().astype(np.float64), self.w.dtype, what)
        np.testing.assert_allclose(self.dbg[1]["mass"].cpu().numpy(), self.dbg[0]["mass"].cpu().numpy(),
                                   rtol=self.H.MASS_RTOL[self.w.dtype], atol=1e-7, err_msg=what)


def test_noalloc_matches_decode_step_two_calls_in_a_row_second_smaller(H):
    from paper_2412_16187_amd import binding as B, synth
    # first: 2 units x 3300 slots, each unit's attention split over many slot ranges whose partial
    # states, local selection keys and hand-over words live in the scratch; second, smaller: 1 unit
    # x 700 slots with kept tokens and two code words
    big = synth.LLAMA8B_DECODE.scaled(n_layers=1, n_kv_heads=2, budget=3300, n_prompt=3400, n_decode=6,
                                      seed=501)
    small = synth.LLAMA8B_DECODE.scaled(n_layers=1, n_kv_heads=1, budget=700, n_prompt=690, n_decode=14,
                                        hash_bits=64, n_sink=4, n_recent=10, seed=502)
    assert B.lshe_decode_plan(B.make_config(128, 32, 2, 4, 1, 1, 3300, "bf16")) == \
        "attn_local_kernel + merge_local_kernel"
    tb, ts = _Twin(H, big), _Twin(H, small)
    for i in range(small.n_decode):
        if i < big.n_decode:
            tb.step_reference(i)
        ts.step_reference(i)
        # the two calls under test, back to back on one stream with nothing between them
        if i < big.n_decode:
            tb.step_noalloc(i)
        ts.step_noalloc(i)
        if i < big.n_decode:
            tb.compare("big, step %d" % i)
        ts.compare("small, step %d" % i)


def test_noalloc_single_kernel_plan_and_groups_of_eight(H):
    from paper_2412_16187_amd import synth
    # one workgroup per unit (needs no scratch at all), then groups of 8 query heads (select, then
    # two attention workgroups per unit) on fewer units
    for kw in (dict(batch=2, n_layers=8, n_kv_heads=8, budget=150, n_prompt=260, n_decode=4),
               dict(batch=1, n_layers=2, n_kv_heads=3, budget=640, n_prompt=700, n_decode=4, gqa_group=8)):
        tw = _Twin(H, synth.LLAMA8B_DECODE.scaled(seed=503, **kw))
        for i in range(tw.w.n_decode):
            tw.step_reference(i)
            tw.step_noalloc(i)
            tw.compare("%s step %d" % (kw, i))


def test_noalloc_rejects_configurations_beyond_its_scratch(H):
    import torch
    from paper_2412_16187_amd import binding as B
    from paper_2412_16187_amd.state import DeviceCache
    # groups of 8 query heads on 1024 units: 1024 x 8 x 130 floats of partial state > 2 MiB
    dc = DeviceCache(4, 32, 8, 8, 128, 32, 600, "bf16")
    assert B.lshe_workspace_bytes(dc.cfg, 0) > B.LSHE_BUILTIN_SCRATCH_BYTES
    dc.n_valid.fill_(5)
    snap = dc.snapshot()
    q = torch.zeros((dc.units, 8, 128), dtype=torch.bfloat16, device=dc.device)
    k = torch.zeros((dc.units, 128), dtype=torch.bfloat16, device=dc.device)
    pos = torch.full((4,), 5, dtype=torch.int32, device=dc.device)
    rc = B.lshe_decode_step_noalloc(dc.cfg, dc.R_dev, q, k, k, pos, dc.K, dc.V, dc.code, dc.slot_pos,
                                    dc.n_valid, dc.out, dc.evicted, None, None, None, check=False)
    assert rc == B.LSHE_SCRATCH_EXCEEDED
    assert "scratch" in B.strerror(rc)
    torch.cuda.synchronize()
    for x, y in zip(snap, dc.snapshot()):
        assert torch.equal(x, y)
    with pytest.raises(B.LsheError):
        B.lshe_decode_step_noalloc(dc.cfg, dc.R_dev, q, k, k, pos, dc.K, dc.V, dc.code, dc.slot_pos,
                                   dc.n_valid, dc.out, dc.evicted, None, None, None)
