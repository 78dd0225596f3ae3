"""CPU-side checks of the C-ABI library: it loads, exports every declared symbol, sizes
follow the closed forms, and argument errors are reported before any device work."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2412_16187_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2412_16187_amd import build
        build.build(verbose=False)
    return B.lib()


def test_exports_every_declared_symbol(lib):
    header = open(os.path.join(ROOT, "include", "lshe.h")).read()
    declared = set(re.findall(r"\b(lshe_[a-z_]+)\s*\(", header))
    assert declared == set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_struct_layout_matches_header():
    header = open(os.path.join(ROOT, "include", "lshe.h")).read()
    body = header[header.index("typedef struct lshe_config {"):header.index("} lshe_config;")]
    fields = re.findall(r"int32_t\s+(\w+);", body)
    assert fields == [f[0] for f in B.lshe_config._fields_]
    assert C.sizeof(B.lshe_config) == 4 * len(fields)


def test_version_and_strerror(lib):
    assert "gfx950" in B.version()
    assert B.strerror(0) == "ok"
    assert "workspace" in B.strerror(B.LSHE_WORKSPACE_TOO_SMALL)


def _cfg(**kw):
    base = dict(head_dim=128, hash_bits=32, n_kv_heads=8, gqa_group=4, n_layers=32, batch=1,
                budget=2048, dtype="bf16")
    base.update(kw)
    return B.make_config(**base)


def test_decode_plan_names(lib):
    # the five benchmark configurations, then the edges of the one-wave-select form
    assert B.lshe_decode_plan(_cfg()) == "decode_fused_solo_kernel"
    assert B.lshe_decode_plan(_cfg(batch=32, budget=1024)) == "decode_fused_kernel"
    assert B.lshe_decode_plan(_cfg(n_layers=1, budget=9830)) == "attn_local_kernel + merge_small_kernel"
    assert B.lshe_decode_plan(_cfg(n_layers=1, budget=3072)) == "attn_local_kernel + merge_small_kernel"
    assert B.lshe_decode_plan(_cfg(n_layers=1, n_kv_heads=1, budget=3073)) == "attn_local_kernel + merge_local_kernel"  # 49 ranges
    assert B.lshe_decode_plan(_cfg(n_layers=1, n_kv_heads=2, budget=9830)) == "attn_local_kernel + merge_local_kernel"  # 128 ranges
    assert B.lshe_decode_plan(_cfg(n_layers=1, n_kv_heads=4, gqa_group=1, hash_bits=16, budget=256,
                                   dtype="f32")) == "decode_fused_kernel"
    assert B.lshe_decode_plan(_cfg(hash_bits=64)) == "decode_fused_solo_kernel"          # 4096 words
    assert B.lshe_decode_plan(_cfg(hash_bits=64, budget=2052)) == "decode_fused_kernel"  # too many
    assert B.lshe_decode_plan(_cfg(budget=2049)) == "decode_fused_kernel"                # not whole vectors
    assert B.lshe_decode_plan(_cfg(budget=1020)) == "decode_fused_kernel"                # too short
    assert B.lshe_decode_plan(_cfg(gqa_group=8)) == "select_kernel + attn_kernel"       # heads shared out
    assert B.lshe_decode_plan(_cfg(gqa_group=8, budget=512)) == "decode_fused_kernel"   # launch-bound anyway
    assert B.lshe_decode_plan(_cfg(n_layers=1, n_kv_heads=1, budget=600)) == "attn_local_kernel + merge_small_kernel"
    assert B.lshe_decode_plan(_cfg(n_layers=1, n_kv_heads=1, budget=600, gqa_group=8)) == "attn_local_kernel + merge_small_kernel"
    assert B.lshe_decode_plan(_cfg(head_dim=96)) is None


def test_prefill_plan_names(lib):
    # which kernels a prompt compression runs: the matrix-core eviction from 8 hash bits and 512
    # slots up, the vector-ALU form below, the code table in global memory when it exceeds LDS
    mfma = "hash_rows_kernel x2 + evict_mfma_kernel + gather_kernel"
    valu = "hash_rows_kernel x2 + evict_lds_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(), 4096) == mfma
    assert B.lshe_prefill_plan(_cfg(batch=8, hash_bits=64, budget=2458), 8192) == mfma
    assert B.lshe_prefill_plan(_cfg(n_layers=1, budget=9830), 32768) == mfma
    assert B.lshe_prefill_plan(_cfg(hash_bits=8), 4096) == mfma
    assert B.lshe_prefill_plan(_cfg(hash_bits=7), 4096) == valu
    assert B.lshe_prefill_plan(_cfg(budget=511), 4096) == valu
    assert B.lshe_prefill_plan(_cfg(n_layers=1, budget=50000), 60000) == \
        "hash_rows_kernel x2 + evict_global_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(), 2048) == "hash_rows_kernel + fill_positions_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(), 0) == "fill_positions_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(policy="l2"), 4096) == "norm_rows_kernel + evict_l2_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(policy="l2"), 100) == "norm_rows_kernel + fill_positions_kernel + gather_kernel"
    assert B.lshe_prefill_plan(_cfg(policy="l2", budget=41500), 50000) is None
    assert B.lshe_prefill_plan(_cfg(), -1) is None
    assert B.lshe_prefill_plan(_cfg(head_dim=96), 4096) is None


def test_config_validation(lib):
    assert B.lshe_check_config(_cfg()) == B.LSHE_OK
    assert B.lshe_check_config(None) == B.LSHE_INVALID_ARG
    for bad in (dict(hash_bits=0), dict(hash_bits=65), dict(gqa_group=0), dict(budget=0),
                dict(budget=1 << 20), dict(dtype=7), dict(n_sink=-1), dict(n_layers=0),
                dict(n_sink=2000, n_recent=48), dict(head_dim=0), dict(policy=2)):
        assert B.lshe_check_config(_cfg(**bad)) == B.LSHE_INVALID_ARG, bad
    for unsup in (dict(head_dim=96), dict(gqa_group=3)):
        assert B.lshe_check_config(_cfg(**unsup)) == B.LSHE_UNSUPPORTED, unsup


def test_sizes_closed_form(lib):
    c = _cfg()
    assert B.lshe_projection_bytes(c) == 32 * 128 * 2
    assert B.lshe_projection_bytes(_cfg(hash_bits=64, dtype="f32")) == 64 * 128 * 4
    assert B.lshe_code_cache_bytes(c) == 32 * 8 * 2048 * 4
    assert B.lshe_workspace_bytes(c, 0) >= 256 * 4
    # prefill workspace holds the key codes and the codes of the queries of tokens >= C
    n = 4096
    need = 256 * n * 4 + 256 * 4 * (n - 2048) * 4
    assert B.lshe_workspace_bytes(c, n) >= need
    assert B.lshe_projection_bytes(_cfg(hash_bits=0)) == 0
    # L2-norm policy: one word per slot whatever the hash width; R keeps its own size
    l2 = _cfg(hash_bits=64, policy="l2")
    assert B.lshe_check_config(l2) == B.LSHE_OK
    assert B.lshe_code_cache_bytes(l2) == 32 * 8 * 2048 * 4
    assert B.lshe_projection_bytes(l2) == 64 * 128 * 2


def test_hash_table_overhead_matches_paper_figures(lib):
    # Section 4.7: 80 layers x 8 KV heads x batch 8 x (8192 * 50%) slots -> 20/40/80 MB at
    # 8/16/32 bits when bits are packed.  Whole uint32 words are stored here, so 32 bits give
    # the paper's figure exactly and fewer bits never exceed the 32-bit figure.
    path = os.path.join(os.path.dirname(__file__), "golden", "hash_table_overhead.txt")
    rows = [l.split() for l in open(path) if l.strip() and not l.startswith("#")]
    for layers, heads, batch, seq, frac, bits, mb in rows:
        c = _cfg(n_layers=int(layers), n_kv_heads=int(heads), batch=int(batch),
                 budget=int(int(seq) * float(frac)), hash_bits=int(bits))
        got = B.lshe_code_cache_bytes(c)
        if int(bits) == 32:
            assert got == float(mb) * 2 ** 20
        assert got == 80 * 2 ** 20


def test_argument_errors_enqueue_nothing(lib):
    c = _cfg()
    one = np.zeros(64, dtype=np.uint8)   # host memory: never dereferenced on an error path
    # NULL required pointers
    assert B.lshe_init_projection(c, 0, None, None, stream=0, check=False) == B.LSHE_INVALID_ARG
    assert B.lshe_hash_keys(c, None, one, 4, one, stream=0, check=False) == B.LSHE_INVALID_ARG
    assert B.lshe_hash_keys(c, one, one, -1, one, stream=0, check=False) == B.LSHE_INVALID_ARG
    assert B.lshe_hash_keys(c, None, None, 0, None, stream=0, check=False) == B.LSHE_OK
    args = [one] * 5
    rc = B.lshe_decode_step(c, one, one, one, one, one, *args, one, None, None, None, None, None,
                            workspace_bytes=0, stream=0, check=False)
    assert rc == B.LSHE_INVALID_ARG
    # short workspace
    raw = np.zeros(2048, dtype=np.uint8)
    off = (-raw.ctypes.data) % 256
    ws = raw[off:off + 1024]
    rc = B.lshe_decode_step(c, one, one, one, one, one, *args, one, None, None, None, None, ws,
                            workspace_bytes=16, stream=0, check=False)
    assert rc == B.LSHE_WORKSPACE_TOO_SMALL
    rc = B.lshe_prefill_compress(c, one, one, one, one, 4096, one, one, one, one, one, None, ws,
                                 workspace_bytes=1024, stream=0, check=False)
    assert rc == B.LSHE_WORKSPACE_TOO_SMALL
    # prompt longer than the budget needs queries
    rc = B.lshe_prefill_compress(c, one, one, one, None, 4096, one, one, one, one, one, None, ws,
                                 workspace_bytes=1 << 40, stream=0, check=False)
    assert rc == B.LSHE_INVALID_ARG
    rc = B.lshe_prefill_compress(c, one, one, one, one, -1, one, one, one, one, one, None, ws,
                                 workspace_bytes=1 << 40, stream=0, check=False)
    assert rc == B.LSHE_INVALID_ARG
    # bad config reaches every entry point
    bad = _cfg(hash_bits=99)
    assert B.lshe_hash_keys(bad, one, one, 4, one, stream=0, check=False) == B.LSHE_INVALID_ARG
    with pytest.raises(B.LsheError):
        B.lshe_hash_keys(bad, one, one, 4, one, stream=0)


def test_l2_policy_refuses_tables_beyond_lds_before_any_launch(lib):
    # the comparator's prompt stage keeps its table of norms in one CU's LDS: budgets beyond
    # 32,768 slots are reported as unsupported, and nothing is enqueued (the pointers here are
    # host memory)
    one = np.zeros(64, dtype=np.uint8)
    raw = np.zeros(2048, dtype=np.uint8)
    ws = raw[(-raw.ctypes.data) % 256:][:1024]
    for budget, kept, n_prompt, want in ((41500, (0, 0), 41600, B.LSHE_UNSUPPORTED),
                                          (32769, (4, 10), 32800, B.LSHE_UNSUPPORTED),
                                          (32768, (4, 10), 32800, None),
                                          (41500, (0, 0), 41500, None),      # no eviction needed
                                          (41500, (0, 0), 41600, "hash")):   # HashEvict has a kernel
        c = _cfg(budget=budget, n_sink=kept[0], n_recent=kept[1], n_kv_heads=1, n_layers=1, batch=1,
                 policy=B.LSHE_POLICY_HASH if want == "hash" else B.LSHE_POLICY_L2NORM)
        rc = B.lshe_prefill_compress(c, one, one, one, one, n_prompt, one, one, one, one, one, None, ws,
                                     workspace_bytes=16, stream=0, check=False)
        # the cases that are supported stop at the next check (workspace too small): still no launch
        assert rc == (want if isinstance(want, int) else B.LSHE_WORKSPACE_TOO_SMALL)
    assert B.lshe_key_norms(_cfg(), None, 4, one, stream=0, check=False) == B.LSHE_INVALID_ARG
    assert B.lshe_key_norms(_cfg(), None, 0, None, stream=0, check=False) == B.LSHE_OK
    rc = B.lshe_decode_step_noalloc(_cfg(hash_bits=0), *([one] * 11), None, None, None, None, stream=0,
                                    check=False)
    assert rc == B.LSHE_INVALID_ARG


def test_bench_refuses_more_than_one_gpu_and_a_machine_without_one():
    # the benchmark is a one-GPU program: asked for more it says so and exits non-zero before
    # touching a GPU; without a GPU it fails loudly instead of falling back to anything
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0 and "ONE GPU" in p.stderr and p.stdout.strip() == ""
    if not os.path.exists("/dev/kfd"):
        p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--steps", "1", "--warmup", "0"],
                           capture_output=True, text=True, timeout=300)
        assert p.returncode != 0 and "no GPU" in p.stderr and p.stdout.strip() == ""


def test_binding_fails_loudly_without_the_library():
    # the product path has no CPU fallback: with the HIP library missing every call raises
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = ("import sys; sys.path.insert(0, %r)\n"
            "from paper_2412_16187_amd import binding as B\n"
            "B.LIB_PATH = B.LIB_PATH + '.absent'\n"
            "try:\n"
            "    B.version()\n"
            "except RuntimeError as e:\n"
            "    assert 'no CPU fallback' in str(e); print('raised')\n" % root)
    p = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=120)
    assert p.returncode == 0 and p.stdout.strip() == "raised", p.stderr
