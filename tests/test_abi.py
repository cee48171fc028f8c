"""The C-ABI library loads and exports every symbol the public header declares (no GPU
needed, no compute calls), and the host-side validation rejects bad configurations."""
import ctypes as C
import os
import re

import pytest

from paper_2003_03477_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "shadowsync.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ss_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    lib = binding.load()
    names = _declared()
    assert len(names) >= 20
    for n in names:
        assert hasattr(lib, n), f"{n} declared in shadowsync.h but not exported"
    assert sorted(binding.EXPORTS) == names


def _cfg(**kw):
    rows = kw.pop("rows", [1000] * 4)
    bot = kw.pop("bot", [13, 64, 16])
    top = kw.pop("top", [26, 64, 1])
    keep = dict(rows=(C.c_int64 * len(rows))(*rows), bot=(C.c_int32 * len(bot))(*bot),
                top=(C.c_int32 * len(top))(*top))
    args = dict(num_tables=len(rows), emb_dim=16, num_dense=13, n_bot=len(bot), n_top=len(top),
                num_replicas=2, max_batch=128, max_ids=4096, num_worker_slots=1, mlp_prec=0,
                lr_dense=0.01, lr_emb=0.01, adagrad_eps=1e-8, seed=1)
    args.update(kw)
    cfg = binding.ss_config(args["num_tables"], keep["rows"], args["emb_dim"], args["num_dense"],
                            args["n_bot"], keep["bot"], args["n_top"], keep["top"],
                            args["num_replicas"], args["max_batch"], args["max_ids"],
                            args["num_worker_slots"], args["mlp_prec"], args["lr_dense"],
                            args["lr_emb"], args["adagrad_eps"], args["seed"])
    return cfg, keep


def test_workspace_size_and_validation_on_host():
    lib = binding.load()
    cfg, keep = _cfg()
    n = lib.ss_workspace_bytes(C.byref(cfg))
    tables = 4000 * 16 * 4
    assert n > tables and n % 256 == 0
    cfg2, keep2 = _cfg(num_worker_slots=3)
    assert lib.ss_workspace_bytes(C.byref(cfg2)) > n
    for bad in (dict(top=[27, 64, 1]), dict(emb_dim=12), dict(bot=[13, 64, 8]),
                dict(num_replicas=0), dict(max_ids=0), dict(top=[26, 64, 2]),
                dict(rows=[0, 5, 5, 5])):
        cfgb, keepb = _cfg(**bad)
        assert lib.ss_workspace_bytes(C.byref(cfgb)) == 0, bad
        assert lib.ss_last_error(None)
    # widest digit of the backward's radix sort: 0 (default), 8, 9 or 10
    for bits, ok in ((0, True), (8, True), (9, True), (10, True), (7, False), (11, False), (-1, False)):
        cfgs, keeps = _cfg()
        cfgs.sort_digit_bits = bits
        assert (lib.ss_workspace_bytes(C.byref(cfgs)) == n) == ok, bits
    ctx = C.c_void_p()
    assert lib.ss_init(C.byref(cfg), None, n, C.byref(ctx)) == -1  # SS_EINVAL: null workspace
    # raw sync entry point rejects malformed arguments before touching the device
    assert lib.ss_sync_round(0, 0, 16, 16, 256, 256, None, None, 0.1, 1.0, 0.0, None) == -1
    assert lib.ss_sync_round(0, 2, 15, 16, 256, 256, None, None, 0.1, 1.0, 0.0, None) == -1
    assert lib.ss_sync_round(2, 2, 16, 16, 256, None, 256, None, 0.1, 1.0, 0.0, None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", "/nonexistent/libshadowsync.so")
    with pytest.raises(RuntimeError):
        binding.load()


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU: `bench.py --gpus N` with N > 1 exits with a message."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "ONE GPU" in r.stderr


def test_workspace_layout_covers_the_bf16_mlp_paths():
    """Host-side layout only (no GPU): the fused and the layer-wise bf16 configurations and a
    model without hidden top layer all produce a workspace size; an unknown mlp_path and a
    bf16 model too large for 32-bit operand indexing are rejected."""
    from paper_2003_03477_amd import binding, synth
    import ctypes as C
    lib = binding.load()

    def size(wl, mlp_path):
        rows = (C.c_int64 * len(wl.rows))(*wl.rows)
        bot = (C.c_int32 * len(wl.bot_dims))(*wl.bot_dims)
        top = (C.c_int32 * len(wl.top_dims))(*wl.top_dims)
        cfg = binding.ss_config(len(wl.rows), rows, wl.emb_dim, wl.bot_dims[0], len(wl.bot_dims), bot,
                                len(wl.top_dims), top, wl.num_replicas, wl.batch, 400000, 2,
                                binding.SS_BF16, 0.01, 0.01, 1e-8, 1, 0, mlp_path)
        return lib.ss_workspace_bytes(C.byref(cfg))

    mid = synth.mid()
    fused = size(mid, 0)
    layerwise = size(mid, 1)
    no_hidden = size(mid.scaled(top_dims=(100, 1)), 0)
    assert fused > 0 and layerwise > 0 and no_hidden > 0
    assert layerwise != fused
    assert size(mid, 7) == 0
    assert size(mid.scaled(batch=1 << 20, top_dims=(100, 4096, 1)), 0) == 0


def test_metrics_and_pace_reject_bad_arguments_without_a_device():
    lib = binding.load()
    assert lib.ss_metrics_read(None, 0, None) == -1
    assert lib.ss_metrics_reset(None, 0) == -1
    assert lib.ss_shadow_pace(None, 10) == -1
