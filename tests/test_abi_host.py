"""Host-only checks of the C ABI: the library loads, exports every symbol the header declares, and rejects bad
arguments before touching a device.  No GPU needed, no kernels launched."""
import ctypes as C
import os
import re

import pytest

from paper_2509_18362_amd import binding as b
from paper_2509_18362_amd import synth

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "mtp_draft.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mtp_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = declared_functions()
    assert set(names) == set(b.EXPORTS)
    lib = C.CDLL(b.LIB_PATH)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    for code in b.STATUS:
        assert b.mtp_status_string(code) != "unknown status"
    assert b.mtp_status_string(-99) == "unknown status"


def test_workspace_bytes_and_config_validation():
    cfg = b.make_config(synth.SEVEN_B, 1, 2112, 3)
    n1 = b.mtp_workspace_bytes(cfg)
    assert n1 > 0 and n1 % 256 == 0
    cfg64 = b.make_config(synth.SEVEN_B, 64, 32832, 5)
    assert b.mtp_workspace_bytes(cfg64) > n1
    assert b.mtp_workspace_bytes(b.make_config(synth.TINY, 1, 192, 3)) > 0
    bad = [dict(d_model=100), dict(head_dim=96), dict(n_kv_heads=3), dict(d_ffn=100), dict(max_batch=0),
           dict(max_batch=513), dict(max_draft_steps=0), dict(kv_capacity=2), dict(rope_theta=0.0), dict(n_kv_heads=1)]
    for kw in bad:
        c = b.make_config(synth.SEVEN_B, 1, 2112, 3)
        for k, v in kw.items():
            setattr(c, k, v)
        assert b.mtp_workspace_bytes(c) == 0, kw


def test_init_rejects_bad_arguments_on_the_host():
    cfg = b.make_config(synth.TINY, 1, 192, 3)
    need = b.mtp_workspace_bytes(cfg)
    fake = {n: 0x1000 for n in b.WEIGHT_FIELDS}  # never dereferenced: every check below fails first
    st, h = b.mtp_draft_init(cfg, {**fake, "w_o": None}, [], [], 0x10000, need)
    assert (st, h) == (-1, None)
    st, _ = b.mtp_draft_init(cfg, fake, [], [], None, need)
    assert st == -1
    st, _ = b.mtp_draft_init(cfg, {**fake, "w_q": 0x1008}, [], [], 0x10000, need)
    assert st == -2
    st, _ = b.mtp_draft_init(cfg, fake, [], [], 0x10000, need - 1)
    assert st == -7
    badcfg = b.make_config(synth.TINY, 1, 192, 3)
    badcfg.head_dim = 48
    st, _ = b.mtp_draft_init(badcfg, fake, [], [], 0x10000, need)
    assert st == -3
    st, _ = b.mtp_draft_init(cfg, fake, [0x2000], [0], 0x10000, need)  # empty id list
    assert st == -6
    st, _ = b.mtp_draft_init(cfg, fake, [0x2000], [synth.TINY.vocab_size + 1], 0x10000, need)
    assert st == -6


def test_calls_reject_null_handle():
    assert b.mtp_draft_steps(None, 1, 1, -1, 16, 16, 16, 16, 16, None, 16, None, None) == -1
    assert b.mtp_accept(None, 1, 1, 16, 16, 0, 16, 16, 16, 16) == -1
    assert b.mtp_poll_error(None) == -1
    assert b.mtp_set_timing(None, 1) == -1
    assert b.mtp_last_draft_ms(None) < 0
    b.mtp_draft_destroy(None)


def test_one_hip_runtime_in_the_process():
    """The library must bind to the HIP runtime PyTorch has loaded, whatever the import order of the caller: a
    second copy of the runtime in the process finds no device."""
    paths = set()
    for line in open("/proc/self/maps"):
        if "libamdhip64" in line:
            paths.add(os.path.realpath(line.split()[-1]))
    assert len(paths) == 1, paths


def test_draft_length_sweep_model_matches_the_printed_tau():
    """tau at K = 3 from the paper's per-position acceptance is the printed 2.73 (tests/golden/paper_values.txt);
    with free drafting the speed-up equals tau, and it falls once a draft step costs more than it brings."""
    from paper_2509_18362_amd import ksweep
    cond = ksweep.conditional_rates(7)
    assert abs(ksweep.expected_tokens(3, cond) - 2.73) < 1e-9
    assert abs(cond[0] - 0.81) < 1e-12 and abs(cond[1] - 0.56 / 0.81) < 1e-12 and cond[3] == cond[2]
    free = ksweep.sweep(0.0, 0.0, 1.0)
    assert all(abs(r["speedup_vs_plain_decoding"] - r["tau"]) < 1e-12 for r in free)
    costly = ksweep.sweep(0.5, 0.0, 1.0)
    best = max(costly, key=lambda r: r["speedup_vs_plain_decoding"])["K"]
    assert best < 7 and costly[-1]["speedup_vs_plain_decoding"] < costly[best - 1]["speedup_vs_plain_decoding"]
