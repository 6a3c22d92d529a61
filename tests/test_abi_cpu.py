"""CPU-only checks of the C ABI: the library loads, exports every symbol the header
declares, and its host-side validation returns the documented error codes before
anything is launched (no GPU is touched by these tests)."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def oqm():
    lib = os.path.join(ROOT, "paper_2510_18269_amd", "libtom_oqm.so")
    if not os.path.exists(lib):
        from paper_2510_18269_amd import build
        build.build()
    from paper_2510_18269_amd import oqm as m
    return m


def test_every_declared_symbol_is_exported(oqm):
    text = ""
    inc = os.path.join(ROOT, "include")
    for name in sorted(os.listdir(inc)):
        if name.endswith(".h"):
            text += open(os.path.join(inc, name)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    declared = set(re.findall(r"\b(tom_[a-z0-9_]+)\s*\(", text))
    assert {"tom_oqm_quantize_append", "tom_oqm_score_groups", "tom_oqm_topk",
            "tom_oqm_dequant_gather"} <= declared
    for sym in declared:
        assert hasattr(oqm.lib, sym), f"{sym} is declared in include/ but not exported"
    assert declared == set(oqm.EXPORTS)


def test_sizes_follow_the_documented_layout(oqm):
    cfg = oqm.make_config(28, 4, 28, 128, 196, 64, 1024)
    s = oqm.tom_oqm_query_sizes(cfg)
    tiles = 28 * 2 * 1024 * 4
    assert s.codes == tiles * 196 * 128 // 2
    assert s.meta == tiles * 196 * 2 * 2 * 4
    assert s.keys == 28 * 1024 * 4 * 128 * 4


@pytest.mark.parametrize("field,value,status", [
    ("head_dim", 100, "INVALID"), ("qgroup", 48, "INVALID"), ("qgroup", 4, "UNSUPPORTED"),
    ("bits", 3, "INVALID"), ("bits", 8, "INVALID"), ("n_q_heads", 27, "INVALID"),
    ("group_tokens", 0, "INVALID"), ("capacity_groups", 0, "INVALID"), ("in_dtype", 7, "INVALID"),
    ("sim", 2, "INVALID"), ("qaxis", 5, "INVALID"), ("meta_dtype", 2, "UNSUPPORTED"),
    ("meta_dtype", 9, "INVALID")])
def test_bad_configurations_are_rejected(oqm, field, value, status):
    cfg = oqm.make_config(2, 4, 28, 128, 196, 64, 16)
    setattr(cfg, field, value)
    with pytest.raises(oqm.TomError) as e:
        oqm.tom_oqm_create(cfg)
    want = oqm.TOM_ERR_INVALID_ARG if status == "INVALID" else oqm.TOM_ERR_UNSUPPORTED
    assert e.value.status == want and oqm.tom_last_error()


def test_host_side_validation_before_any_launch(oqm):
    cfg = oqm.make_config(2, 2, 4, 64, 16, 32, 8)
    h = oqm.tom_oqm_create(cfg)
    try:
        fake = 0x1000                                    # never dereferenced: every call below fails first
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, None, (1, 1, 1, 1))
        assert e.value.status == oqm.TOM_ERR_NOT_BOUND
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_bind(h, fake, fake + 4, fake)           # misaligned
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        oqm.tom_oqm_bind(h, fake, fake, fake)
        assert oqm.tom_oqm_num_groups(h) == 0
        st = (2 * 2 * 16 * 64, 2 * 16 * 64, 16 * 64, 64)
        with pytest.raises(oqm.TomError) as e:           # over capacity: nothing is evicted
            oqm.tom_oqm_quantize_append(h, 0, 2, 9, fake, fake, None, st)
        assert e.value.status == oqm.TOM_ERR_CAPACITY and oqm.tom_oqm_num_groups(h) == 0
        with pytest.raises(oqm.TomError) as e:           # layer range
            oqm.tom_oqm_quantize_append(h, 1, 2, 1, fake, fake, None, st)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        with pytest.raises(oqm.TomError) as e:           # stride not a multiple of 16 bytes
            oqm.tom_oqm_quantize_append(h, 0, 2, 1, fake, fake, None, (st[0], st[1], st[2], 65))
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_quantize_append(h, 0, 2, 1, None, fake, None, st)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        # no-ops succeed without touching the GPU
        assert oqm.tom_oqm_quantize_append(h, 0, 2, 0, fake, fake, None, st) == 0
        oqm.tom_oqm_score_groups(h, 0, 2, fake, 1, fake, 0, q_dtype=oqm.TOM_F32)   # T == 0
        oqm.tom_oqm_dequant_gather(h, 0, 2, fake, 4, 0, fake, fake)                # k_eff == 0
        with pytest.raises(oqm.TomError):
            oqm.tom_oqm_dequant_gather(h, 0, 2, fake, 4, 5, fake, fake)            # k_eff > k
        with pytest.raises(oqm.TomError):
            oqm.tom_oqm_dequant_gather(h, 0, 3, fake, 4, 1, fake, fake)            # layers
        # checkpoint restore: the counter can be set within capacity only
        oqm.tom_oqm_set_num_groups(h, 8)
        assert oqm.tom_oqm_num_groups(h) == 8
        with pytest.raises(oqm.TomError):
            oqm.tom_oqm_set_num_groups(h, 9)
        with pytest.raises(oqm.TomError) as e:           # score needs a workspace
            oqm.tom_oqm_score_groups(h, 0, 2, fake, 1, fake, 8, q_dtype=oqm.TOM_F32)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG and "workspace" in str(e.value)
        with pytest.raises(oqm.TomError):                # stride shorter than T
            oqm.tom_oqm_score_groups(h, 0, 2, fake, 1, fake, 7, q_dtype=oqm.TOM_F32)
        oqm.tom_oqm_reset(h)
        assert oqm.tom_oqm_num_groups(h) == 0
    finally:
        oqm.tom_oqm_destroy(h)


def test_assemble_and_retrieve_validation(oqm):
    cfg = oqm.make_config(2, 2, 4, 64, 16, 32, 8)
    h = oqm.tom_oqm_create(cfg)
    try:
        fake = 0x1000
        oqm.tom_oqm_bind(h, fake, fake, fake)
        with pytest.raises(oqm.TomError) as e:           # negative prefix
            oqm.tom_oqm_assemble_active(h, 0, 2, fake, 4, 1, -1, None, None, fake, fake)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        with pytest.raises(oqm.TomError) as e:           # only one system tensor
            oqm.tom_oqm_assemble_active(h, 0, 2, fake, 4, 1, 3, fake, None, fake, fake)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        with pytest.raises(oqm.TomError) as e:           # misaligned system tensor
            oqm.tom_oqm_assemble_active(h, 0, 2, fake, 4, 1, 3, fake + 2, fake, fake, fake)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
        # nothing to do: no groups selected and no prefix to copy
        oqm.tom_oqm_assemble_active(h, 0, 2, fake, 4, 0, 3, None, None, fake, fake)
        # one-call retrieval on an empty store: k_eff = 0, nothing launched
        assert oqm.tom_oqm_retrieve(h, 0, 2, fake, 1, 4, fake, 8, fake, fake, fake, None,
                                    q_dtype=oqm.TOM_F32) == 0
        # with groups stored, every step is validated before the first launch:
        # the gather's k_out is missing, so the score kernel must not have been queued
        oqm.tom_oqm_set_num_groups(h, 8)
        nbytes = oqm.tom_oqm_score_workspace_bytes(h, 2, 1, oqm.TOM_SCORE_AUTO)

        class FakeWs:                                    # a workspace that is never touched
            is_cuda = True
            def data_ptr(self): return fake
            def numel(self): return nbytes
            def element_size(self): return 1
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_retrieve(h, 0, 2, fake, 1, 4, fake, 8, fake, None, fake, FakeWs(),
                                 q_dtype=oqm.TOM_F32)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG and "k_out" in str(e.value)
    finally:
        oqm.tom_oqm_destroy(h)


def test_retrieve_noalloc_checks_sizes_and_arguments_on_the_host(oqm):
    """The entry point that allocates nothing: its scratch limit and the validation of all
    three steps are host-side and come before the first GPU call."""
    assert oqm.tom_oqm_static_scratch_bytes() == 8 << 20
    cfg = oqm.make_config(2, 4, 28, 128, 16, 64, 8)
    h = oqm.tom_oqm_create(cfg)
    try:
        fake = 0x1000
        oqm.tom_oqm_bind(h, fake, fake, fake)
        # empty store: k_eff = 0, nothing launched, the scratch is not even looked up
        assert oqm.tom_oqm_retrieve_noalloc(h, 0, 2, fake, 1, 4, fake, 8, fake, fake, fake,
                                            q_dtype=oqm.TOM_F32) == 0
        oqm.tom_oqm_set_num_groups(h, 8)
        # 2 layers x 2048 query tokens x 512 channels of float64 = 16 MiB on the matrix-core path
        assert oqm.tom_oqm_score_workspace_bytes(h, 2, 2048, oqm.TOM_SCORE_TOKEN_GEMM) > 8 << 20
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_retrieve_noalloc(h, 0, 2, fake, 2048, 4, fake, 8, fake, fake, fake,
                                         path=oqm.TOM_SCORE_TOKEN_GEMM, q_dtype=oqm.TOM_F32)
        assert e.value.status == oqm.TOM_ERR_UNSUPPORTED and "static scratch" in str(e.value)
        # the same query on the mean-query path fits; the missing k_out is then found by the
        # validation pass, before any device is asked for the array's address
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_retrieve_noalloc(h, 0, 2, fake, 2048, 4, fake, 8, fake, None, fake,
                                         path=oqm.TOM_SCORE_MEAN_QUERY, q_dtype=oqm.TOM_F32)
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG and "k_out" in str(e.value)
    finally:
        oqm.tom_oqm_destroy(h)


def test_launch_size_limits_are_reported_before_any_launch(oqm):
    """Shapes whose 1-D grids would not fit are refused as UNSUPPORTED by the validation pass."""
    fake = 0x1000
    # append: n_frames * n_layers * H_k * (G + 1) must stay below 2^31
    cfg = oqm.make_config(1000, 8, 8, 64, 60000, 32, 70000)
    h = oqm.tom_oqm_create(cfg)
    try:
        oqm.tom_oqm_bind(h, fake, fake, fake)
        st = (1000 * 8 * 60000 * 64, 8 * 60000 * 64, 60000 * 64, 64)
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_quantize_append(h, 0, 1000, 60000, fake, fake, None, st)
        assert e.value.status == oqm.TOM_ERR_UNSUPPORTED and "2^31" in str(e.value)
        # gather: k_eff * ceil(G / 3) along one grid dimension
        oqm.tom_oqm_set_num_groups(h, 70000)
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_dequant_gather(h, 0, 1, fake, 200000, 140000, fake, fake)   # 140000 groups x 20000 chunks
        assert e.value.status == oqm.TOM_ERR_UNSUPPORTED and "2^31" in str(e.value)
    finally:
        oqm.tom_oqm_destroy(h)
    cfg = oqm.make_config(1, 1, 1, 8, 200000, 8, 40000)       # G = 200000: up to 66667 chunks per tile
    h = oqm.tom_oqm_create(cfg)
    try:
        oqm.tom_oqm_bind(h, fake, fake, fake)
        oqm.tom_oqm_set_num_groups(h, 40000)
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_dequant_gather(h, 0, 1, fake, 40000, 40000, fake, fake)
        assert e.value.status == oqm.TOM_ERR_UNSUPPORTED and "2^31" in str(e.value)
        # astronomically large strides are refused, not multiplied
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_quantize_append(h, 0, 1, 0 + 1, fake, fake, None, (2 ** 62, 8, 8, 8))
        assert e.value.status in (oqm.TOM_ERR_INVALID_ARG, oqm.TOM_ERR_CAPACITY)
    finally:
        oqm.tom_oqm_destroy(h)
    # a configuration whose storage could not be addressed in 64 bits
    with pytest.raises(oqm.TomError) as e:
        oqm.tom_oqm_create(oqm.make_config(2 ** 31 - 1, 4, 4, 2048, 1000, 64, 2 ** 31 - 1))
    assert e.value.status == oqm.TOM_ERR_UNSUPPORTED


def test_two_bit_sizes(oqm):
    cfg = oqm.make_config(28, 4, 28, 128, 50, 64, 100, bits=2)
    s = oqm.tom_oqm_query_sizes(cfg)
    tiles = 28 * 2 * 100 * 4
    assert s.codes == tiles * 50 * 32 and s.meta == tiles * 50 * 2 * 2 * 4


def test_bf16_metadata_sizes(oqm):
    cfg = oqm.make_config(28, 4, 28, 128, 196, 64, 1024, meta_dtype=oqm.TOM_BF16)
    s = oqm.tom_oqm_query_sizes(cfg)
    assert s.meta == 28 * 2 * 1024 * 4 * 196 * 2 * 2 * 2      # half of the float32 pairs


def test_token_axis_sizes(oqm):
    cfg = oqm.make_config(28, 4, 28, 128, 50, 64, 100, qaxis=oqm.TOM_QAXIS_TOKENS)
    cfg.qgroup = 7                                        # ignored on the token axis
    s = oqm.tom_oqm_query_sizes(cfg)
    tiles = 28 * 2 * 100 * 4
    assert s.codes == tiles * 50 * 64 and s.meta == tiles * 128 * 2 * 4


def test_workspace_size(oqm):
    cfg = oqm.make_config(28, 4, 28, 128, 196, 64, 16)
    h = oqm.tom_oqm_create(cfg)
    try:
        small = oqm.tom_oqm_score_workspace_bytes(h, 28, 32, oqm.TOM_SCORE_MEAN_QUERY)
        big = oqm.tom_oqm_score_workspace_bytes(h, 28, 32, oqm.TOM_SCORE_TOKEN_GEMM)
        assert small >= 28 * (512 + 4) * 8 and small < 28 * 520 * 8 + 64
        assert big - small == 28 * 32 * 512 * 8
        assert oqm.tom_oqm_score_workspace_bytes(h, 28, 32, oqm.TOM_SCORE_AUTO, True) == big
        assert oqm.tom_oqm_score_workspace_bytes(h, 28, 0) == 0
    finally:
        oqm.tom_oqm_destroy(h)


def test_topk_argument_checks_and_k_eff(oqm):
    k_eff = oqm.tom_oqm_topk(0x1000, 16, 0, 10, 64, 0x1000)        # no rows: nothing launched
    assert k_eff == 10
    assert oqm.tom_oqm_topk(0x1000, 16, 3, 0, 4, 0x1000) == 0      # nothing stored yet
    for bad in (dict(k=0), dict(n_groups=-1), dict(score_stride=5), dict(order=3)):
        args = dict(score_stride=16, n_rows=1, n_groups=10, k=4, order=0)
        args.update(bad)
        with pytest.raises(oqm.TomError) as e:
            oqm.tom_oqm_topk(0x1000, args["score_stride"], args["n_rows"], args["n_groups"],
                             args["k"], 0x1000, order=args["order"])
        assert e.value.status == oqm.TOM_ERR_INVALID_ARG
    with pytest.raises(oqm.TomError) as e:
        oqm.tom_oqm_topk(0x1000, 10000, 1, 10000, 5000, 0x1000, order=oqm.TOM_ORDER_SCORE_DESC)
    assert e.value.status == oqm.TOM_ERR_UNSUPPORTED


def test_k_from_budget_matches_the_supplement_formula(oqm, oracle):
    for B, G, T in [(12544, 196, 1000), (12544, 50, 10 ** 6), (12544, 50, 7), (1, 50, 10), (0, 50, 10)]:
        assert oqm.tom_oqm_k_from_budget(B, G, T) == oracle.k_from_budget(B, G, T * G)


def test_bench_refuses_more_than_one_gpu():
    """The path has no collectives: `bench.py --gpus N` with N > 1 exits with a message and
    touches no GPU (the check comes before torch is imported)."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=60)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr and r.stdout.strip() == ""


def test_product_and_oracle_do_not_reference_each_other():
    """The library and its binding never touch the oracle (there is no CPU fallback), and the
    oracle never touches the library: only the seeded input generator is common to both."""
    pkg = os.path.join(ROOT, "paper_2510_18269_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.lower(), f"{f} mentions the oracle"
    for f in os.listdir(os.path.join(ROOT, "oracle")):
        if f.endswith((".py", ".c", ".h")):
            text = open(os.path.join(ROOT, "oracle", f)).read()
            assert "paper_2510_18269_amd" not in text and "libtom_oqm" not in text and "tom_oqm.h" not in text, f
    header = open(os.path.join(ROOT, "include", "tom_oqm.h")).read()
    assert "tomref" not in header


def test_last_error_is_per_thread(oqm):
    """tom_last_error returns the message of the calling thread's own last failure."""
    import threading
    out = {}
    barrier = threading.Barrier(2)

    def worker(name, field, value, needle):
        kw = dict(n_layers=1, n_kv_heads=2, n_q_heads=2, head_dim=64, group_tokens=4, qgroup=32, capacity=2)
        cfg = oqm.make_config(kw["n_layers"], kw["n_kv_heads"], kw["n_q_heads"], kw["head_dim"],
                              kw["group_tokens"], kw["qgroup"], kw["capacity"])
        setattr(cfg, field, value)
        sizes = oqm.tom_oqm_sizes_t()
        for _ in range(200):
            st = oqm.lib.tom_oqm_query_sizes(C.byref(cfg), C.byref(sizes))
            try:
                barrier.wait(timeout=30)        # both threads have failed before either reads
            except threading.BrokenBarrierError:
                out.setdefault(name, "partner stopped")
                break
            msg = oqm.tom_last_error()
            if st == oqm.TOM_OK or needle not in msg:
                out[name] = (st, msg)
                barrier.abort()
                break
        else:
            out[name] = "ok"

    a = threading.Thread(target=worker, args=("a", "head_dim", 12, "head_dim"))
    b = threading.Thread(target=worker, args=("b", "bits", 3, "bits"))
    a.start(); b.start(); a.join(); b.join()
    assert out == {"a": "ok", "b": "ok"}, out
