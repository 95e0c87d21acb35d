"""Host-side checks that need no GPU: the library loads, exports every symbol the header
declares, sizes its buffers, and rejects bad arguments / out-of-order calls (dry context)."""
import ctypes as C
import os
import re

import numpy as np
import pytest

from paper_2412_04757_amd import (LtriConfig, LtriContext, LtriError, config_from_workload,
                                  load_library, library_path, EXPORTED_SYMBOLS)
from workloads import CONFIGS

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    """Every function declared by the headers under include/ (the product boundary and the bench helpers)."""
    names = set()
    inc = os.path.join(ROOT, "include")
    for fn in sorted(os.listdir(inc)):
        if fn.endswith(".h"):
            text = open(os.path.join(inc, fn)).read()
            text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
            names |= set(re.findall(r"\b(ltri_[a-z_]+)\s*\(", text))
    return sorted(names)


def test_library_exports_every_declared_symbol():
    lib = load_library()
    declared = _declared_symbols()
    assert len(declared) >= 20
    for name in declared:
        assert hasattr(lib, name), name
    assert sorted(EXPORTED_SYMBOLS) == declared
    assert b"gfx950" in lib.ltri_version()


def test_workspace_sizes_and_bad_configs():
    lib = load_library()
    for name in ("cfg1", "cfg2", "cfg3"):
        cfg = config_from_workload(CONFIGS[name], theta=1.0)
        sb, cb = C.c_size_t(), C.c_size_t()
        assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0
        assert sb.value > 0 and cb.value > 0 and sb.value % 256 == 0
    # cfg4: 32 layers of index memory stay modest next to the KV arenas
    cfg = config_from_workload(CONFIGS["cfg4"], theta=1.0)
    sb, cb = C.c_size_t(), C.c_size_t()
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0
    kv = 2 * 32 * 8 * 262144 * 128 * 2
    assert sb.value < kv / 8
    bad = [dict(head_dim=96), dict(dtype=7), dict(n_kv_heads=3), dict(chunk_max=4096), dict(chunk_max=0),
           dict(max_tokens=0), dict(seg_map=3), dict(phi=-0.1), dict(window=-1), dict(n_layers=0),
           dict(max_spans=70000)]
    for kw in bad:
        cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0)
        for k, v in kw.items():
            setattr(cfg, k, v)
        assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == -1, kw
    # dynamic span index vectors: parameters are checked only in that mode
    cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0, rep_mode=1, lam=3.0, index_min=2, index_max=16, ratio_mode=2)
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0
    mean_scratch = C.c_size_t()
    cfg0 = config_from_workload(CONFIGS["cfg1"], theta=1.0)
    assert lib.ltri_workspace_bytes(C.byref(cfg0), C.byref(sb), C.byref(mean_scratch)) == 0
    assert cb.value > mean_scratch.value                       # the row log-sum-exp pieces
    for kw in (dict(rep_mode=2), dict(lam=-1.0), dict(lam=float("nan")), dict(index_min=-1), dict(index_max=1),
               dict(ratio_mode=3)):
        cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0, rep_mode=1, lam=3.0, index_min=2, index_max=16)
        for k, v in kw.items():
            setattr(cfg, k, v)
        assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == -1, kw
    # retrieval by memory units: at most a chunk long, at most 8192 units in a full stream
    for ut, ok in ((0, True), (32, True), (256, True), (257, False), (-1, False)):
        cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0, unit_tokens=ut)
        assert (lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0) == ok, ut
    cfg = config_from_workload(CONFIGS["cfg3"], theta=1.0, unit_tokens=16)            # 131072 / 16 units
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == -1
    cfg = config_from_workload(CONFIGS["cfg3"], theta=1.0, unit_tokens=128, theta_quantile=0.9)
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0
    cfg.theta_quantile = 1.5
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == -1
    # a budget of index vectors per block needs dynamic index vectors and memory units
    for kw, ok in ((dict(rep_mode=1, unit_tokens=128, index_block_max=12), True), (dict(rep_mode=1, index_block_max=12), False),
                   (dict(unit_tokens=128, index_block_max=12), False), (dict(rep_mode=1, unit_tokens=128, index_block_max=-1), False)):
        cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0, **kw)
        assert (lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0) == ok, kw
    cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0, lam=-5.0, ratio_mode=9)    # ignored with mean keys
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == 0
    cfg = config_from_workload(CONFIGS["cfg1"], theta=1.0)
    cfg.dtype = 1            # bf16 with head_dim 64 is not supported
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb), C.byref(cb)) == -1
    out = C.c_void_p()
    assert lib.ltri_create(C.byref(cfg), None, None, None, None, None, C.byref(out)) == -1
    assert lib.ltri_strerror(-3).decode().startswith("token or span capacity")


def test_collaborative_retrieval_call_rules_in_dry_mode():
    w = CONFIGS["cfg1"]
    ctx = LtriContext(config_from_workload(w, max_tokens=1024, theta=1.0, n_layers=3), None, dry=True)
    ctx.append_chunk(1, 0, 1, 256)
    with pytest.raises(LtriError) as e:
        ctx.retrieve_collaborative(1, 0, 1, _FakeQ(256), [1.0, 1.0])
    assert e.value.status == -1                      # spans are retrieved: nothing to vote on
    ctx.close()
    ctx = LtriContext(config_from_workload(w, max_tokens=1024, theta=1.0, n_layers=3, unit_tokens=64), None, dry=True)
    for layer in range(3):
        ctx.append_chunk(layer, 0, 1, 256)
    with pytest.raises(LtriError) as e:
        ctx.retrieve_collaborative(1, 0, 1, _FakeQ(256), [0.5, 1.0])
    assert e.value.status == -2                      # layer 0 votes but has no selection yet
    ctx.retrieve_collaborative(1, 0, 1, _FakeQ(256), [0.0, 1.0])        # weight 0: layer 0 takes no part
    ctx.retrieve(0, 0, 1, _FakeQ(256))
    ctx.retrieve_collaborative(2, 0, 1, _FakeQ(256), [0.5, 0.25, 1.0])
    ctx.attend(2, 0, 1, _FakeQ(256))
    with pytest.raises(LtriError) as e:
        ctx.retrieve_collaborative(2, 0, 1, _FakeQ(256), [0.5, -0.25, 1.0])
    assert e.value.status == -1
    ctx.append_chunk(0, 0, 1, 256)                   # layer 0 moves on: its selection is for another chunk
    with pytest.raises(LtriError) as e:
        ctx.retrieve_collaborative(2, 0, 1, _FakeQ(256), [0.5, 0.25, 1.0])
    assert e.value.status == -2
    ctx.close()
    big = LtriContext(config_from_workload(CONFIGS["cfg3"], theta=1.0, n_layers=2, unit_tokens=16,
                                           max_tokens=131072 - 64), None, dry=True)
    big.append_chunk(1, 0, 1, 2048)
    with pytest.raises(LtriError) as e:
        big.retrieve_collaborative(1, 0, 1, _FakeQ(2048), [0.0, 1.0])   # 4096 units and more
    assert e.value.status == -1
    big.close()


class _FakeQ:
    """Stands in for a device tensor in dry mode: only the shape and a non-null address are used."""
    def __init__(self, n_q):
        self.shape = (1, n_q, 4, 64)

    def data_ptr(self):
        return 4096


def test_call_order_and_limits_in_dry_mode():
    cfg = config_from_workload(CONFIGS["cfg1"], max_tokens=1000, theta=1.0)
    ctx = LtriContext(cfg, None, dry=True)
    with pytest.raises(LtriError) as e:
        ctx.retrieve(0, 0, 1, _FakeQ(256))
    assert e.value.status == -2                      # retrieve before any append
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(0, 0, 1, 257)
    assert e.value.status == -1                      # n_new > chunk_max
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(0, 0, 1, 0)
    assert e.value.status == -1
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(1, 0, 1, 16)
    assert e.value.status == -1                      # layer out of range
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(0, 0, 2, 16)
    assert e.value.status == -1                      # sequence range
    with pytest.raises(LtriError) as e:
        ctx.retrieve_persistent(0, 0, 1)
    assert e.value.status == -2                      # nothing appended
    ctx.append_chunk(0, 0, 1, 256)
    assert ctx.token_count(0, 0) == 256
    with pytest.raises(LtriError) as e:
        ctx.attend(0, 0, 1, _FakeQ(256))
    assert e.value.status == -2                      # attend before retrieve
    with pytest.raises(LtriError) as e:
        ctx.retrieve_persistent(0, 0, 1)
    assert e.value.status == -2                      # no earlier selection to keep
    with pytest.raises(LtriError) as e:
        ctx.retrieve(0, 0, 1, _FakeQ(128))
    assert e.value.status == -2                      # n_q differs from the appended chunk
    ctx.retrieve(0, 0, 1, _FakeQ(256))
    ctx.attend(0, 0, 1, _FakeQ(256))
    ctx.append_chunk(0, 0, 1, 256)
    with pytest.raises(LtriError) as e:
        ctx.attend(0, 0, 1, _FakeQ(256))             # the selection belongs to the previous chunk
    assert e.value.status == -2
    ctx.force_selection(0, 0, 0, [3, 1, 1])
    ctx.attend(0, 0, 1, _FakeQ(256))                 # one KV head: forced selection is enough
    ctx.append_chunk(0, 0, 1, 256)
    ctx.retrieve_persistent(0, 0, 1)                 # the earlier selection is kept for the new chunk
    ctx.attend(0, 0, 1, _FakeQ(256))
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(0, 0, 1, 256)               # 768 + 256 > 1000
    assert e.value.status == -3 and "max_tokens" in str(e.value)
    ctx.append_chunk(0, 0, 1, 232)
    assert ctx.token_count(0, 0) == 1000
    ctx.reset(0)
    assert ctx.token_count(0, 0) == 0
    with pytest.raises(LtriError) as e:
        ctx.span_count(0, 0, 0)                      # no device data in a dry context
    assert e.value.status == -2
    # caller-supplied boundaries are validated on the host
    for bad in ([0, 5, 5, 16], [1, 16], [0, 8], [0, 16, 8]):
        with pytest.raises(LtriError) as e:
            ctx.append_chunk_with_spans(0, 0, 16, [np.array(bad)])
        assert e.value.status == -1, bad
    ctx.append_chunk_with_spans(0, 0, 16, [np.array([0, 4, 16])])
    assert ctx.token_count(0, 0) == 16
    with pytest.raises(LtriError) as e:
        ctx.get_theta(0, 0, 0)
    assert e.value.status == -2                      # a dry context selects no threshold
    with pytest.raises(LtriError) as e:
        ctx.get_theta(0, 0, 9)
    assert e.value.status == -1                      # KV head out of range
    ctx.close()


def test_whole_step_call_rules_in_dry_mode():
    """ltri_step is append + retrieve + attend for the host logic: it advances the stream, leaves a selection
    behind, and fails where any of the three would."""
    cfg = config_from_workload(CONFIGS["cfg1"], max_tokens=600, theta=1.0)
    ctx = LtriContext(cfg, None, dry=True)
    ctx.step(0, 0, 1, None, None, _FakeQ(256))
    assert ctx.token_count(0, 0) == 256
    ctx.attend(0, 0, 1, _FakeQ(256))                 # the step left a selection for this chunk
    ctx.step(0, 0, 1, None, None, _FakeQ(100))
    assert ctx.token_count(0, 0) == 356
    with pytest.raises(LtriError) as e:
        ctx.step(0, 0, 1, None, None, _FakeQ(257))   # longer than chunk_max
    assert e.value.status == -1
    with pytest.raises(LtriError) as e:
        ctx.step(0, 0, 1, None, None, _FakeQ(245))   # 356 + 245 > max_tokens
    assert e.value.status == -3
    assert ctx.token_count(0, 0) == 356              # a failed step appends nothing
    with pytest.raises(LtriError) as e:
        ctx.step(0, 1, 1, None, None, _FakeQ(16))    # sequence out of range
    assert e.value.status == -1
    ctx.close()


def test_attend_static_rules_in_dry_mode():
    """ltri_attend_static: the call order rules of ltri_attend, and LTRI_ECAPACITY when the partial results of the
    call would not fit the library's own 2 MiB (checked on the host, before anything is enqueued)."""
    class Q:
        def __init__(self, n_seqs, n_q):
            self.shape = (n_seqs, n_q, 32, 128)

        def data_ptr(self):
            return 4096
    w = CONFIGS["cfg5"]
    ctx = LtriContext(config_from_workload(w, max_tokens=4096, theta=1.0, n_seqs=16), None, dry=True)
    with pytest.raises(LtriError) as e:
        ctx.attend_static(0, 0, 16, Q(16, 1), None)
    assert e.value.status == -2                      # nothing appended yet
    ctx.append_chunk(0, 0, 16, 1)
    with pytest.raises(LtriError) as e:
        ctx.attend_static(0, 0, 16, Q(16, 1), None)
    assert e.value.status == -2                      # no selection for the chunk
    ctx.retrieve(0, 0, 16, Q(16, 1))
    ctx.attend_static(0, 0, 16, Q(16, 1), None)      # the decode batch of config 5 fits (1.1 MB)
    ctx.append_chunk(0, 0, 2, 4)
    ctx.retrieve(0, 0, 2, Q(2, 4))
    with pytest.raises(LtriError) as e:
        ctx.attend_static(0, 0, 2, Q(2, 4), None)    # 2 x 32 heads x 16 splits x 4 rows x 130 floats = 2.13 MB
    assert e.value.status == -3 and "2097152" in str(e.value)
    ctx.attend(0, 0, 2, Q(2, 4))                     # the context's scratch takes it
    ctx.append_chunk(0, 0, 16, 2048)
    ctx.retrieve(0, 0, 16, Q(16, 2048))
    ctx.attend_static(0, 0, 16, Q(16, 2048), None)   # long chunks keep no partial results
    ctx.close()


def test_host_offloaded_kv_rules_in_dry_mode():
    """kv_offload: the device pools are part of `state`, the flag is 0 or 1, and an append must bring the rows."""
    lib = load_library()
    w = CONFIGS["cfg3"]
    sb0, sb1, cb = C.c_size_t(), C.c_size_t(), C.c_size_t()
    cfg = config_from_workload(w, theta=1.0)
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb0), C.byref(cb)) == 0
    cfg = config_from_workload(w, theta=1.0, kv_offload=1)
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb1), C.byref(cb)) == 0
    # per KV head: 4 initial rows + a ring of 8192 (>= 4096 + 2 x 2048) + 2048 mirror rows + the list capacity, K and V
    rows = 4 + 8192 + 2048 + (((4 + 8192 + 4096 + 63) // 64) * 64 + 64)
    assert sb1.value - sb0.value >= 2 * 8 * rows * 256
    assert sb1.value - sb0.value <= 2 * 8 * rows * 256 + 8 * rows * 4 + 4096
    cfg.kv_offload = 2
    assert lib.ltri_workspace_bytes(C.byref(cfg), C.byref(sb1), C.byref(cb)) == -1
    ctx = LtriContext(config_from_workload(CONFIGS["cfg1"], max_tokens=1024, theta=1.0, kv_offload=1), None, dry=True)
    with pytest.raises(LtriError) as e:
        ctx.append_chunk(0, 0, 1, 256)                   # rows "already in the arena": there is no device arena
    assert e.value.status == -1
    with pytest.raises(LtriError) as e:
        ctx.step(0, 0, 1, None, None, _FakeQ(256))
    assert e.value.status == -1
    ctx.append_chunk(0, 0, 1, 256, k_chunk=_FakeQ(256), v_chunk=_FakeQ(256))
    ctx.retrieve(0, 0, 1, _FakeQ(256))
    ctx.attend(0, 0, 1, _FakeQ(256))
    ctx.step(0, 0, 1, _FakeQ(256), _FakeQ(256), _FakeQ(256))
    assert ctx.token_count(0, 0) == 512
    ctx.close()


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N > 1 exits with a message before it touches a device."""
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""
