"""The C-ABI library loads, exports every symbol the header declares, and rejects bad arguments on the host
(no GPU needed: validation happens before anything is launched)."""
import ctypes as C
import os
import re

import pytest

import paper_2602_08404_amd as tm
from paper_2602_08404_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = "".join(open(os.path.join(ROOT, "include", f)).read() for f in sorted(os.listdir(os.path.join(ROOT, "include"))) if f.endswith(".h"))
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(team_moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    lib = binding.lib()
    names = declared_symbols()
    assert set(names) == set(binding.EXPORTS)
    for n in names:
        assert getattr(lib, n) is not None


def test_status_strings():
    assert tm.status_string(0) == "ok"
    for s in (-1, -2, -3, -4, -5, 99):
        assert isinstance(tm.status_string(s), str) and tm.status_string(s)


def test_workspace_size_grows_with_tokens_and_covers_intermediates():
    small = tm.team_moe_workspace_size(tm.make_config(2048, 768, 128, 8, "bf16", 1, 32))
    big = tm.team_moe_workspace_size(tm.make_config(2048, 768, 128, 8, "bf16", 1, 128))
    assert big > small
    A = 32 * 8
    assert small >= A * 768 * 2 + A * 2048 * 4 + 4 * A * 4 + 129 * 4 + 128 * 4 + 4
    assert small % 256 == 0


@pytest.mark.parametrize("kw,status", [
    (dict(hidden=2048, inter=768, num_experts=128, top_k=0), -1),
    (dict(hidden=2048, inter=768, num_experts=4, top_k=8), -1),
    (dict(hidden=2048, inter=768, num_experts=512, top_k=8), -2),
    (dict(hidden=2048, inter=768, num_experts=128, top_k=32), -2),
    (dict(hidden=2000, inter=768, num_experts=128, top_k=8), -2),
    (dict(hidden=2048, inter=700, num_experts=128, top_k=8), -2),
    (dict(hidden=2048, inter=768, num_experts=128, top_k=8, max_tokens=4096), -2),
    (dict(hidden=2048, inter=768, num_experts=128, top_k=8, max_tokens=0), -1),
])
def test_bad_configs_are_rejected(kw, status):
    kw = dict(dict(dtype="bf16", renormalize=1, max_tokens=32), **kw)
    cfg = tm.make_config(**kw)
    with pytest.raises(tm.TeamMoeError) as e:
        tm.team_moe_workspace_size(cfg)
    assert e.value.status == status


def test_bad_call_arguments_are_rejected_before_any_launch():
    lib = binding.lib()
    cfg = tm.make_config(2048, 768, 128, 8, "bf16", 1, 32)
    fake = C.c_void_p(0x1000)          # aligned, never dereferenced: every call below fails validation first
    odd = C.c_void_p(0x1004)
    st = 0
    # NULL required pointers
    assert lib.team_moe_route(C.byref(cfg), None, 8, fake, None, fake, fake, None, None, 0, st) == -1
    assert lib.team_moe_build_dispatch(C.byref(cfg), None, 8, fake, fake, fake, fake, fake, None, 0, st) == -1
    assert lib.team_moe_combine(C.byref(cfg), fake, fake, None, 8, fake, st) == -1
    assert lib.team_moe_expert_ffn(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, fake, None, fake, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, None, fake, 1 << 30, st) == -1
    # token count out of range
    assert lib.team_moe_route(C.byref(cfg), fake, 0, fake, None, fake, fake, None, None, 0, st) == -1
    assert lib.team_moe_route(C.byref(cfg), fake, 33, fake, None, fake, fake, None, None, 0, st) == -1
    # no logits_out and no workspace to keep the scores in
    assert lib.team_moe_route(C.byref(cfg), fake, 8, fake, None, fake, fake, None, None, 0, st) == -3
    assert lib.team_moe_route(C.byref(cfg), fake, 8, fake, None, fake, fake, None, fake, 64, st) == -3
    # misaligned tensor
    assert lib.team_moe_route(C.byref(cfg), odd, 8, fake, None, fake, fake, None, None, 0, st) == -1
    # workspace missing / too small / misaligned
    assert lib.team_moe_layer_forward(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, fake, None, 0, st) == -3
    assert lib.team_moe_layer_forward(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, fake, fake, 1024, st) == -3
    assert lib.team_moe_layer_forward(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, fake, odd, 1 << 30, st) == -3
    assert lib.team_moe_expert_ffn(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, fake, fake, fake, fake, 16, st) == -3
    # two-round routing: token classes and a full workspace are required
    assert lib.team_moe_route_two_round(C.byref(cfg), fake, 8, fake, None, None, None, fake, fake, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_route_two_round(C.byref(cfg), fake, 8, fake, fake, None, None, fake, fake, None, None, 0, st) == -3
    assert lib.team_moe_route_two_round(C.byref(cfg), fake, 8, fake, fake, None, None, fake, fake, fake, fake, 1024, st) == -3
    assert lib.team_moe_route_two_round(C.byref(cfg), fake, 40, fake, fake, None, None, fake, fake, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward_two_round(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, None, None, fake, fake,
                                                1 << 30, st) == -1
    assert lib.team_moe_layer_forward_two_round(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, None, None, fake, None,
                                                0, st) == -3
    # token classification: required pointers, sizes, threshold
    f32 = C.c_float
    assert lib.team_moe_classify_tokens(None, fake, 32, 32, None, 32, f32(0.7), 3, fake, st) == -1
    assert lib.team_moe_classify_tokens(fake, fake, 32, 32, None, 32, f32(0.7), 3, None, st) == -1
    assert lib.team_moe_classify_tokens(fake, fake, 32, 0, None, 32, f32(0.7), 3, fake, st) == -1
    assert lib.team_moe_classify_tokens(fake, fake, 32, 32, None, 33, f32(0.7), 3, fake, st) == -1      # more tokens than rows
    assert lib.team_moe_classify_tokens(fake, fake, 32, 32, None, 32, f32(0.7), -1, fake, st) == -1
    assert lib.team_moe_classify_tokens(fake, fake, 32, 32, None, 32, f32(float("nan")), 3, fake, st) == -1
    # layer over live rows: the index list and a positive row count are required, one routing mode per call
    rows_args = (8, fake, fake, fake, fake)
    assert lib.team_moe_layer_forward_rows(C.byref(cfg), fake, fake, 32, None, *rows_args, None, None, None, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward_rows(C.byref(cfg), fake, fake, 0, fake, *rows_args, None, None, None, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward_rows(C.byref(cfg), fake, fake, 32, fake, *rows_args, fake, fake, None, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward_rows(C.byref(cfg), fake, fake, 32, fake, *rows_args, None, None, None, None, None, 0, st) == -3
    # repeated rows: same validation as the plain layer (the optional outputs may be NULL)
    assert lib.team_moe_layer_forward_unique_rows(C.byref(cfg), None, 8, fake, fake, fake, fake, None, fake, None, None, fake, 1 << 30, st) == -1
    assert lib.team_moe_layer_forward_unique_rows(C.byref(cfg), fake, 8, fake, fake, fake, fake, None, fake, None, None, fake, 1024, st) == -3
    # 8-bit weights: scale tables required and 4-byte aligned; bf16 configuration with hidden 1024/2048 and inter % 256 == 0
    w8_tail = (fake, fake, 1 << 30, st)
    assert lib.team_moe_layer_forward_w8(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, None, fake, None, *w8_tail) == -1
    assert lib.team_moe_layer_forward_w8(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, C.c_void_p(0x1002), fake, None, *w8_tail) == -1
    assert lib.team_moe_layer_forward_w8(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, fake, fake, None, fake, None, 0, st) == -3
    for bad_cfg in (tm.make_config(2048, 640, 128, 8, "bf16", 1, 32), tm.make_config(512, 768, 128, 8, "bf16", 1, 32),
                    tm.make_config(2048, 768, 128, 8, "f32", 1, 32)):
        assert lib.team_moe_layer_forward_w8(C.byref(bad_cfg), fake, 8, fake, fake, fake, fake, fake, fake, fake, None, *w8_tail) == -2
        assert lib.team_moe_expert_ffn_w8(C.byref(bad_cfg), fake, 8, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake, fake,
                                          fake, 1 << 30, st) == -2
    assert lib.team_moe_expert_ffn_w8(C.byref(cfg), fake, 8, fake, fake, fake, fake, fake, fake, fake, fake, fake, None, fake,
                                      fake, 1 << 30, st) == -1
    i64 = C.c_int64
    assert lib.team_moe_dequantize_w8(None, fake, i64(4), i64(64), fake, st) == -1
    assert lib.team_moe_dequantize_w8(fake, fake, i64(4), i64(40), fake, st) == -1          # columns not a multiple of 16
    assert lib.team_moe_dequantize_w8(fake, fake, i64(0), i64(64), fake, st) == -1
    assert lib.team_moe_dequantize_w8(odd, fake, i64(4), i64(64), fake, st) == -1
    # the combined call: combinations that are not supported, stray outputs, bad row counts
    def ex(**kw):
        base = dict(x=0x1000, y=0x1000, T=8, n_rows=0, row_index=None, w_router=0x1000, w_gate=0x1000, w_up=0x1000, w_down=0x1000,
                    workspace=0x1000, ws_bytes=1 << 30, stream=None)
        base.update(kw)
        return lib.team_moe_layer_forward_ex(C.byref(cfg), C.byref(binding.LayerArgs(**base)))
    assert lib.team_moe_layer_forward_ex(C.byref(cfg), None) == -1
    assert ex(expert_mask=0x1000, token_class=0x1000) == -1
    assert ex(unique_rows=2) == -1
    assert ex(row_rep_out=0x1000) == -1
    assert ex(n_activated_out=0x1000) == -1
    assert ex(row_index=0x1000, n_rows=0) == -1
    assert ex(n_rows=16) == -1
    assert ex(reserved=1) == -1
    assert ex(scale_gate=0x1000) == -1                       # all three scale tables or none
    assert ex(workspace=None, ws_bytes=0) == -3
    assert ex(x=None) == -1
    assert ex(ffn_begin_event=0x1000) == -1                  # both events or none
    # the workspace's failure mark: a status area is 256 bytes
    assert lib.team_moe_workspace_status(fake, 128, st) == -3
    assert lib.team_moe_workspace_status(odd, 1 << 20, st) == -3
    # the static-array layer: configurations that do not fit its 16 MiB are rejected before anything else happens
    big = tm.make_config(2048, 512, 256, 8, "bf16", 1, 256)
    assert lib.team_moe_layer_forward_static(C.byref(big), fake, 256, fake, fake, fake, fake, None, fake, st) == -3
    # tuning / testing knobs
    v = C.c_int(0)
    assert lib.team_moe_internal_set(b"no_such_knob", 1) == -1 and lib.team_moe_internal_get(b"no_such_knob", C.byref(v)) == -1
    assert lib.team_moe_internal_get(b"ffn_spin_limit", None) == -1
    assert lib.team_moe_internal_get(b"row_hash_bits", C.byref(v)) == 0 and v.value == 64
    assert lib.team_moe_internal_set(b"row_hash_bits", 3) == 0 and tm.internal_get("row_hash_bits") == 3
    tm.internal_set("row_hash_bits", 64)
    # NULL cfg / NULL size pointer
    assert lib.team_moe_workspace_size(None, C.byref(C.c_size_t())) == -1
    assert lib.team_moe_workspace_size(C.byref(cfg), None) == -1
    bad = tm.make_config(2048, 768, 128, 8, "bf16", 1, 32)
    bad.dtype = 7
    assert lib.team_moe_route(C.byref(bad), fake, 8, fake, None, fake, fake, None, None, 0, st) == -1


def test_product_package_does_not_use_the_oracle():
    """No file of the product package imports, includes, loads or names a path of the oracle."""
    pkg = os.path.join(ROOT, "paper_2602_08404_amd")
    pat = re.compile(r"(import\s+oracle|from\s+oracle|from\s+\.\.?\s*oracle|#include\s+\"[^\"]*oracle|libteam_moe_oracle|oracle/)")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".hpp", ".h", ".cpp")):
                assert not pat.search(open(os.path.join(dirpath, f)).read()), f


def test_bench_refuses_more_than_one_gpu():
    """bench.py --gpus N with N above 1 exits with a message that says so, before anything touches a GPU."""
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
