"""Host-side checks of the C-ABI library: it loads, exports every symbol the header
declares, and rejects bad arguments before touching the GPU (no GPU needed)."""
import ctypes
import os
import re

import pytest

import paper_2203_04738_amd as mg
from paper_2203_04738_amd.binding import MgritGruCfg

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared_symbols():
    text = open(os.path.join(ROOT, "include", "mgrit_gru.h")).read()
    return re.findall(r"MGRIT_API\s+[\w\s\*]+?\b(\w+)\s*\(", text)


def test_library_loads_and_exports_every_declared_symbol():
    names = _declared_symbols()
    assert set(names) >= {"mgrit_gru_forward", "mgrit_gru_backward", "gru_serial_scan",
                          "gru_serial_scan_backward", "mgrit_gru_workspace_bytes"}
    L = mg.lib()
    for n in names:
        assert hasattr(L, n), n


def test_cfg_struct_matches_header_field_order():
    text = open(os.path.join(ROOT, "include", "mgrit_gru.h")).read()
    body = text[text.index("typedef struct {"):text.index("} mgrit_gru_cfg;")]
    fields = []
    for line in body.splitlines():
        m = re.match(r"\s*int32_t\s+([\w,\s]+);", line)
        if m:
            fields += [f.strip() for f in m.group(1).split(",")]
    assert fields == [f for f, _ in MgritGruCfg._fields_]


def _ws(cfg):
    n = ctypes.c_size_t(0)
    rc = mg.lib().mgrit_gru_workspace_bytes(ctypes.byref(cfg), ctypes.byref(n))
    return rc, n.value


def test_workspace_size_and_validation_codes():
    rc, n = _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=3))
    assert rc == 0 and n >= 64 * 2 * 96 * 4
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=4, iters=1))[0] == 0    # coarsest level: 1 step
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=5, iters=1))[0] == -3
    assert _ws(MgritGruCfg(60, 2, 16, 32, cf=4, levels=3, iters=1))[0] == -3
    assert _ws(MgritGruCfg(0, 2, 16, 32))[0] == -2
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=0, levels=2))[0] == -2
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=0))[0] == -2
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=-1))[0] == -2
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, propagator=2))[0] == -4
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, dtype=7))[0] == -4
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, fine_relax=2))[0] == -4
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, flags=8))[0] == 0
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, flags=16))[0] == 0
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, flags=32))[0] == -4
    assert _ws(MgritGruCfg(64, 2, 16, 30, cf=4, levels=2))[0] == -6
    assert _ws(MgritGruCfg(64, 2, 9, 32, cf=4, levels=2))[0] == -6
    # fp32 values as three bf16 terms: widths in multiples of 8, a larger workspace (term arrays)
    assert _ws(MgritGruCfg(64, 2, 16, 36, cf=4, levels=2, dtype=2))[0] == -6
    rc2, n2 = _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=3, dtype=2))
    assert rc2 == 0 and n2 >= n + 18 * 32 * (2 * 32 + 16)
    # both bf16 forms: the same workspace, widths in multiples of 8
    rc3, n3 = _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=3, dtype=3))
    rc1, n1 = _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=3, dtype=1))
    assert rc3 == 0 and rc1 == 0 and n3 == n1
    assert _ws(MgritGruCfg(64, 2, 16, 36, cf=4, levels=2, dtype=3))[0] == -6
    assert _ws(MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, dtype=4))[0] == -4
    assert mg.lib().mgrit_gru_workspace_bytes(None, None) == -1


def test_entry_points_reject_null_and_small_workspace_without_a_gpu():
    L = mg.lib()
    cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1)
    # null data pointers: refused on the host, nothing is launched
    assert L.gru_serial_scan(ctypes.byref(cfg), None, None, None, None, None, None, None,
                             None, 0, None) == -1
    assert L.mgrit_gru_forward(ctypes.byref(cfg), None, None, None, None, None, None, None, None,
                               None, 0, None) == -1
    assert L.mgrit_gru_backward(ctypes.byref(cfg), None, None, None, None, None, None, None, None,
                                None, None, None, None, None, None, 0, None) == -1
    # fake but aligned addresses with a too-small workspace: refused before any launch
    p = 4096
    assert L.mgrit_gru_forward(ctypes.byref(cfg), p, p, p, p, p, p, p, None, p, 16, None) == -5
    assert L.gru_serial_scan(ctypes.byref(cfg), p, p, p, p, p, p, p, p, 16, None) == -5
    # misaligned pointer
    assert L.mgrit_gru_forward(ctypes.byref(cfg), p + 4, p, p, p, p, p, p, None, p, 1 << 30,
                               None) == -6
    # gradients: all four or none
    assert L.mgrit_gru_backward(ctypes.byref(cfg), p, p, p, p, p, p, p, p, None, p, None, None,
                                None, p, 1 << 30, None) == -1


def test_step_loss_entry_points_validate_their_arguments_without_a_gpu():
    L = mg.lib()
    cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1)
    p = 4096
    # the loss array is required
    assert L.mgrit_gru_backward_steps(ctypes.byref(cfg), p, p, p, p, p, p, None, p, None, p, p,
                                      p, p, p, p, 1 << 30, None) == -1
    assert L.gru_serial_scan_backward_steps(ctypes.byref(cfg), p, p, p, p, p, p, None, p, p, p,
                                            p, p, p, p, 1 << 30, None) == -1
    # misaligned loss array or dx
    assert L.mgrit_gru_backward_steps(ctypes.byref(cfg), p, p, p, p, p, p, p + 4, p, None, p, p,
                                      p, p, p, p, 1 << 30, None) == -6
    assert L.mgrit_gru_backward_steps(ctypes.byref(cfg), p, p, p, p, p, p, p, p, None, p, p,
                                      p, p, p + 8, p, 1 << 30, None) == -6
    # too-small workspace: refused before any launch
    assert L.mgrit_gru_backward_steps(ctypes.byref(cfg), p, p, p, p, p, p, p, p, None, p, p,
                                      p, p, p, p, 16, None) == -5


def test_ode_entry_points_validate_their_arguments_without_a_gpu():
    L = mg.lib()
    cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1)
    p = 4096
    dt = ctypes.c_float(0.25)
    assert L.mgrit_ode_forward(ctypes.byref(cfg), dt, None, None, None, None, None, None, None,
                               None, 0, None) == -1
    assert L.ode_serial_scan(ctypes.byref(cfg), dt, p, p, p, p, p, p, p, 16, None) == -5
    assert L.mgrit_ode_forward(ctypes.byref(cfg), dt, p, p, p, p, p, p, None, p, 16, None) == -5
    # step size must be positive and finite
    for bad in (0.0, -1.0, float("nan"), float("inf")):
        assert L.mgrit_ode_forward(ctypes.byref(cfg), ctypes.c_float(bad), p, p, p, p, p, p, None,
                                   p, 1 << 30, None) == -2
    # fp32 operands and no flags only
    for kw in ({"dtype": mg.MGRIT_BF16}, {"dtype": mg.MGRIT_F32_BF16X3},
               {"flags": mg.MGRIT_ZERO_STATE_GUESS}):
        c2 = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, **kw)
        assert L.mgrit_ode_forward(ctypes.byref(c2), dt, p, p, p, p, p, p, None, p, 1 << 30,
                                   None) == -8
    # the propagator field is not read; the hierarchy is checked
    c3 = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, propagator=77)
    assert L.mgrit_ode_forward(ctypes.byref(c3), dt, p, p, p, p, p, p, None, p, 16, None) == -5
    c4 = MgritGruCfg(60, 2, 16, 32, cf=8, levels=2, iters=1)
    assert L.mgrit_ode_forward(ctypes.byref(c4), dt, p, p, p, p, p, p, None, p, 1 << 30,
                               None) == -3


def test_strerror_names_codes():
    assert mg.mgrit_gru_strerror(0) == "ok"
    assert "divide" in mg.mgrit_gru_strerror(-3)
    with pytest.raises(mg.MgritGruError):
        mg.mgrit_gru_workspace_bytes(MgritGruCfg(60, 2, 16, 32, cf=4, levels=3))


def test_bench_refuses_more_than_one_gpu():
    # one GPU only: the bench exits with a message instead of starting ranks
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "--gpus 1" in r.stderr


def test_reuse_flags_are_refused_on_a_workspace_the_library_has_no_record_of():
    """MGRIT_REUSE_PROJECTION / MGRIT_REUSE_COEFFS are checked against a host-side record keyed
    by the workspace pointer; with no matching record the call is refused before any launch."""
    L = mg.lib()
    p = 4096
    ws = 1 << 20                      # an address no call has used as a workspace
    for flags in (mg.MGRIT_REUSE_PROJECTION, mg.MGRIT_REUSE_COEFFS,
                  mg.MGRIT_REUSE_PROJECTION | mg.MGRIT_REUSE_COEFFS):
        cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, flags=flags)
        assert L.mgrit_gru_backward(ctypes.byref(cfg), p, p, p, p, p, p, p, p, None, p, p, p, p,
                                    ws, 1 << 30, None) == mg.MGRIT_E_STATE
        assert L.gru_serial_scan_backward(ctypes.byref(cfg), p, p, p, p, p, p, p, p, p, p, p, p,
                                          ws, 1 << 30, None) == mg.MGRIT_E_STATE
    cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, flags=mg.MGRIT_REUSE_PROJECTION)
    assert L.mgrit_gru_forward(ctypes.byref(cfg), p, p, p, p, p, p, p, None, ws, 1 << 30,
                               None) == mg.MGRIT_E_STATE
    assert "REUSE" in mg.mgrit_gru_strerror(mg.MGRIT_E_STATE)


def test_static_workspace_entry_point_validates_on_the_host():
    L = mg.lib()
    p = 4096
    ok = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1)
    assert L.mgrit_gru_forward_static(ctypes.byref(ok), None, p, p, p, p, p, p, None, None) == -1
    assert L.mgrit_gru_forward_static(None, p, p, p, p, p, p, p, None, None) == -1
    # a problem whose workspace exceeds the fixed array: refused with the workspace code
    big = MgritGruCfg(2048, 32, 1024, 512, cf=4, levels=3, iters=2)
    assert mg.mgrit_gru_workspace_bytes(big) > mg.MGRIT_STATIC_SCRATCH_BYTES
    assert L.mgrit_gru_forward_static(ctypes.byref(big), p, p, p, p, p, p, p, None, None) == -5
    # nothing is kept in or reused from the fixed array across calls
    for flags in (mg.MGRIT_REUSE_PROJECTION, mg.MGRIT_KEEP_COEFFS):
        c = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, flags=flags)
        assert L.mgrit_gru_forward_static(ctypes.byref(c), p, p, p, p, p, p, p, None, None) == -8
    bad = MgritGruCfg(60, 2, 16, 32, cf=4, levels=3, iters=1)
    assert L.mgrit_gru_forward_static(ctypes.byref(bad), p, p, p, p, p, p, p, None, None) == -3
    text = open(os.path.join(ROOT, "include", "mgrit_gru.h")).read()
    m = re.search(r"#define MGRIT_STATIC_SCRATCH_BYTES \((\d+)u << (\d+)\)", text)
    assert int(m.group(1)) << int(m.group(2)) == mg.MGRIT_STATIC_SCRATCH_BYTES


def test_binding_rejects_tensors_whose_size_does_not_match_cfg():
    """The C ABI takes plain pointers; the binding compares every tensor's shape with cfg and
    raises before anything is launched (CPU tensors suffice to reach the shape checks)."""
    import torch
    T, B, D, H = 8, 2, 4, 8
    cfg = MgritGruCfg(T, B, D, H, cf=2, levels=2, iters=3)
    z = lambda *s: torch.zeros(*s)
    good = dict(W=z(3 * H, D), U=z(3 * H, H), b_i=z(3 * H), b_h=z(3 * H), x=z(T, B, D))
    states, ws = z(T + 1, B, H), torch.zeros(1 << 16, dtype=torch.uint8)
    g = (z(3 * H, D), z(3 * H, H), z(3 * H), z(3 * H))

    def fwd(**over):
        a = dict(good, h0=z(B, H), h=states, res=z(3))
        a.update(over)
        mg.mgrit_gru_forward(cfg, a["W"], a["U"], a["b_i"], a["b_h"], a["x"], a["h0"], a["h"],
                             a["res"], ws)

    for over in (dict(h=z(T, B, H)), dict(res=z(2)), dict(x=z(T + 1, B, D)), dict(W=z(3 * H, H)),
                 dict(U=z(H, H)), dict(b_i=z(H)), dict(b_h=z(3 * H + 1)), dict(h0=z(B, H + 1))):
        with pytest.raises(ValueError):
            fwd(**over)
    with pytest.raises(TypeError):       # right sizes, but not device memory
        fwd()
    P = tuple(good.values())
    with pytest.raises(ValueError):      # the step-loss entry point takes dL_dh[(T+1),B,H]
        mg.mgrit_gru_backward_steps(cfg, *P, states, z(B, H), states, z(3), *g, z(T, B, D), ws)
    with pytest.raises(ValueError):      # ... and the terminal-loss one dL_dhT[B,H]
        mg.mgrit_gru_backward(cfg, *P, states, states, states, z(3), *g, ws)
    with pytest.raises(ValueError):
        mg.mgrit_gru_backward_steps(cfg, *P, states, states, states, z(3), *g, z(T, B, H), ws)
    with pytest.raises(ValueError):
        mg.mgrit_gru_backward(cfg, *P, states, z(B, H), states, z(3), g[1], g[1], g[2], g[3], ws)
    with pytest.raises(ValueError):
        mg.gru_serial_scan(cfg, *P, z(B, H), z(T, B, H), ws)
    with pytest.raises(ValueError):
        mg.gru_serial_scan_backward(cfg, *P, states, z(B, H), z(T, B, H), *g, ws)
    with pytest.raises(ValueError):
        mg.mgrit_ode_forward(cfg, 0.1, z(H, D), z(H, D), z(H), z(T, B, D), z(B, H), states, z(3), ws)
    with pytest.raises(ValueError):
        mg.mgrit_gru_forward_static(cfg, *P, z(B, H), z(T, B, H), z(3))


def test_lstm_entry_points_validate_their_arguments_without_a_gpu():
    L = mg.lib()
    cfg = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1)
    p = 4096
    # state pairs (h | c) double the state arrays: a larger workspace than the GRU's
    assert mg.mgrit_lstm_workspace_bytes(cfg) > mg.mgrit_gru_workspace_bytes(cfg)
    assert L.mgrit_lstm_forward(ctypes.byref(cfg), None, None, None, None, None, None, None, None,
                                None, 0, None) == -1
    assert L.lstm_serial_scan(ctypes.byref(cfg), p, p, p, p, p, p, p, p, 16, None) == -5
    assert L.mgrit_lstm_forward(ctypes.byref(cfg), p, p, p, p, p, p, p, None, p, 16, None) == -5
    for kw in ({"dtype": mg.MGRIT_BF16}, {"dtype": mg.MGRIT_F32_BF16X3},
               {"flags": mg.MGRIT_ZERO_STATE_GUESS}):
        c2 = MgritGruCfg(64, 2, 16, 32, cf=4, levels=2, iters=1, **kw)
        assert L.mgrit_lstm_forward(ctypes.byref(c2), p, p, p, p, p, p, p, None, p, 1 << 30,
                                    None) == -8
    c3 = MgritGruCfg(60, 2, 16, 32, cf=8, levels=2, iters=1)
    assert L.mgrit_lstm_forward(ctypes.byref(c3), p, p, p, p, p, p, p, None, p, 1 << 30,
                                None) == -3
    c4 = MgritGruCfg(64, 2, 16, 30, cf=4, levels=2, iters=1)
    assert L.mgrit_lstm_forward(ctypes.byref(c4), p, p, p, p, p, p, p, None, p, 1 << 30,
                                None) == -6
    import torch
    z = lambda *s: torch.zeros(*s)
    with pytest.raises(ValueError):       # the state arrays hold pairs: [(T+1), B, 2H]
        mg.mgrit_lstm_forward(cfg, z(128, 16), z(128, 32), z(128), z(128), z(64, 2, 16), z(2, 64),
                              z(65, 2, 32), z(1), torch.zeros(16, dtype=torch.uint8))
