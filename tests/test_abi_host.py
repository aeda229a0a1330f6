"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, and rejects bad arguments before anything would be launched."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def pkg():
    import paper_2605_02888_amd as p
    from paper_2605_02888_amd import build
    build.build()          # compiles only if a source is newer than the library
    p.load_library()
    return p


def declared_functions():
    text = open(os.path.join(ROOT, "include", "speckv.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(speckv_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls_of_the_path():
    names = declared_functions()
    for n in ("speckv_signals", "speckv_verify", "speckv_verify_greedy", "speckv_select_gamma", "speckv_step", "speckv_sample_draft", "speckv_create", "speckv_destroy",
              "speckv_workspace_bytes", "speckv_last_error", "speckv_row_offsets"):
        assert n in names


def test_library_exports_every_declared_symbol(pkg):
    lib = pkg.load_library()
    for n in declared_functions():
        assert hasattr(lib, n), n


def test_workspace_bytes(pkg):
    assert pkg.workspace_bytes(0, 8) == 0
    assert pkg.workspace_bytes(4, 0) == 0
    assert pkg.workspace_bytes(4, 17) == 0
    a, b = pkg.workspace_bytes(256, 8), pkg.workspace_bytes(512, 8)
    assert 0 < a < b and a % 256 == 0


def _expect(pkg, status, fn, *args, **kw):
    with pytest.raises(pkg.SpecKVError) as e:
        fn(*args, **kw)
    assert pkg.STATUS_NAMES[e.value.status] == status, str(e.value)


def test_argument_errors_are_reported_before_any_launch(pkg):
    h = pkg.SpecKV(device=-1)   # no device: a call that passes validation reports ERR_DEVICE
    ok = pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=4)
    big = 1 << 30
    A = 4096                    # any 16-byte aligned fake address: nothing is dereferenced
    sig = lambda b=ok, d=A, dt=2, ws=A, wsb=big, H=A, c=A, am=None, ag=A: \
        h.signals(b, d, dt, ws, H, c, am, ag, ws_bytes=wsb, stream=0)
    _expect(pkg, "ERR_DEVICE", sig)
    _expect(pkg, "ERR_NULL", sig, d=None)
    _expect(pkg, "ERR_NULL", sig, H=None)
    _expect(pkg, "ERR_DTYPE", sig, dt=7)
    _expect(pkg, "ERR_ALIGN", sig, d=A + 4)
    _expect(pkg, "ERR_ALIGN", sig, ws=A + 8)
    _expect(pkg, "ERR_WORKSPACE", sig, wsb=pkg.workspace_bytes(4, 8) - 1)
    _expect(pkg, "ERR_SHAPE", sig, b=pkg.Batch(B=0, V=100, gamma_max=8, gamma_uniform=4))
    _expect(pkg, "ERR_SHAPE", sig, b=pkg.Batch(B=4, V=0, gamma_max=8, gamma_uniform=4))
    _expect(pkg, "ERR_GAMMA", sig, b=pkg.Batch(B=4, V=100, gamma_max=17, gamma_uniform=4))
    _expect(pkg, "ERR_GAMMA", sig, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=9))
    _expect(pkg, "ERR_GAMMA", sig, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=0))
    _expect(pkg, "ERR_NULL", sig, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma=A))          # ragged without row_off
    _expect(pkg, "ERR_NULL", sig, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=4, row_off=A))

    ver = lambda b=ok, t=A, d=A, tok=A, ws=A, n=A: \
        h.verify(b, t, d, 2, tok, 1, 0, ws, n, A, A, None, None, ws_bytes=big, stream=0)
    _expect(pkg, "ERR_STATE", ver)            # no speckv_signals before it
    _expect(pkg, "ERR_NULL", ver, tok=None)
    _expect(pkg, "ERR_ALIGN", ver, t=A + 2)

    gre = lambda b=ok, t=A, tok=A, ws=A, n=A, wsb=big: \
        h.verify_greedy(b, t, 2, tok, ws, n, A, A, None, None, ws_bytes=wsb, stream=0)
    _expect(pkg, "ERR_DEVICE", gre)           # needs no speckv_signals before it
    _expect(pkg, "ERR_NULL", gre, tok=None)
    _expect(pkg, "ERR_ALIGN", gre, t=A + 2)
    _expect(pkg, "ERR_WORKSPACE", gre, wsb=16)

    mlp = dict(n_in=5, n_hidden=16, W1=A, b1=A, W2=A, b2=A)
    sel = lambda m=mlp, mode=0, H=A, c=A, ag=A, comp=A, out=A: \
        h.select_gamma(ok, m, mode, H, c, ag, comp, out, None, stream=0)
    _expect(pkg, "ERR_DEVICE", sel)
    _expect(pkg, "ERR_SHAPE", sel, m=dict(mlp, n_in=7))
    _expect(pkg, "ERR_SHAPE", sel, m=dict(mlp, n_hidden=65))
    _expect(pkg, "ERR_SHAPE", sel, m=dict(mlp, n_hidden=-1))
    _expect(pkg, "ERR_DTYPE", sel, m=dict(mlp, form=2))
    _expect(pkg, "ERR_DEVICE", sel, m=dict(mlp, form=1))
    _expect(pkg, "ERR_DEVICE", sel, m=dict(mlp, n_hidden=0, W1=None, b1=None))   # no hidden layer: W1, b1 unused
    _expect(pkg, "ERR_NULL", sel, m=dict(mlp, W1=None))
    _expect(pkg, "ERR_SHAPE", sel, m=dict(mlp, n_in=5), mode=1)
    _expect(pkg, "ERR_DTYPE", sel, mode=3)
    _expect(pkg, "ERR_NULL", sel, H=None)
    _expect(pkg, "ERR_NULL", sel, m=dict(mlp, W2=None))
    _expect(pkg, "ERR_NULL", sel, out=None)
    _expect(pkg, "ERR_DEVICE", sel, m=dict(mlp, n_in=7), mode=1, H=None, c=None)

    smp = lambda b=ok, d=A, dt=2, tok=A: h.sample_draft(b, d, dt, 1, 0, 0, tok, None, None, stream=0)
    _expect(pkg, "ERR_DEVICE", smp)
    _expect(pkg, "ERR_NULL", smp, d=None)
    _expect(pkg, "ERR_NULL", smp, tok=None)
    _expect(pkg, "ERR_DTYPE", smp, dt=9)
    _expect(pkg, "ERR_ALIGN", smp, d=A + 2)
    _expect(pkg, "ERR_GAMMA", smp, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=0))

    one = lambda b=ok, m=mlp, mode=0, d=A, t=A, dt=2, tok=A, comp=A, ws=A, wsb=big, H=A, am=None, n=A, gn=A: \
        h.step(b, m, mode, d, t, dt, tok, comp, 1, 0, ws, H, A, am, A, n, A, A, None, None, gn, None,
               ws_bytes=wsb, stream=0)
    _expect(pkg, "ERR_DEVICE", one)           # every check passed
    _expect(pkg, "ERR_NULL", one, d=None)
    _expect(pkg, "ERR_NULL", one, t=None)
    _expect(pkg, "ERR_NULL", one, tok=None)
    _expect(pkg, "ERR_NULL", one, comp=None)
    _expect(pkg, "ERR_NULL", one, H=None)
    _expect(pkg, "ERR_NULL", one, n=None)
    _expect(pkg, "ERR_NULL", one, gn=None)
    _expect(pkg, "ERR_NULL", one, m=dict(mlp, b1=None))
    _expect(pkg, "ERR_DTYPE", one, dt=5)
    _expect(pkg, "ERR_DTYPE", one, mode=2)
    _expect(pkg, "ERR_SHAPE", one, m=dict(mlp, n_in=7))
    _expect(pkg, "ERR_ALIGN", one, d=A + 2)
    _expect(pkg, "ERR_ALIGN", one, t=A + 8)
    _expect(pkg, "ERR_ALIGN", one, ws=A + 4)
    _expect(pkg, "ERR_WORKSPACE", one, wsb=pkg.workspace_bytes(4, 8) - 1)
    _expect(pkg, "ERR_GAMMA", one, b=pkg.Batch(B=4, V=100, gamma_max=8, gamma_uniform=9))
    grd = lambda g: h.step(ok, mlp, 0, A, A, 2, A, A, 1, 0, A, A, A, None, A, A, A, A, None, None, A, None,
                           ws_bytes=big, stream=0, greedy=g)
    _expect(pkg, "ERR_DEVICE", grd, 1)
    _expect(pkg, "ERR_DTYPE", grd, 2)

    # the step on the library's own workspace: same checks, and a batch beyond the array is refused
    sta = lambda b=ok, m=mlp, d=A, tok=A, H=A: \
        h.step_static(b, m, 0, d, A, 2, tok, A, 1, 0, H, A, None, A, A, A, A, None, None, A, None, stream=0)
    _expect(pkg, "ERR_DEVICE", sta)
    _expect(pkg, "ERR_NULL", sta, d=None)
    _expect(pkg, "ERR_NULL", sta, H=None)
    _expect(pkg, "ERR_ALIGN", sta, d=A + 2)
    _expect(pkg, "ERR_SHAPE", sta, m=dict(mlp, n_in=7))
    assert pkg.workspace_bytes(4096, 8) <= pkg.STATIC_WS_BYTES < pkg.workspace_bytes(8192, 8)
    _expect(pkg, "ERR_DEVICE", sta, b=pkg.Batch(B=4096, V=100, gamma_max=8, gamma_uniform=8))
    _expect(pkg, "ERR_WORKSPACE", sta, b=pkg.Batch(B=8192, V=100, gamma_max=8, gamma_uniform=8))
    _expect(pkg, "ERR_WORKSPACE", sta, b=pkg.Batch(B=1 << 20, V=100, gamma_max=16, gamma_uniform=8))
    h.close()


def test_options_round_trip_and_reject_bad_values(pkg):
    h = pkg.SpecKV(device=-1)
    for name, good, bad in (("stats_threads", 512, 100), ("stats_unroll", 4, 8), ("step_tail", 0, 2), ("stats_target_wgs", 4096, 0),
                            ("stats_max_split", 4, 0), ("stats_pipeline", 0, 2), ("stats_nontemporal", 0, 5),
                            ("profile_every", 8, 0), ("stats_wgs_per_cu", 0, 1), ("stats_wgs_per_cu", 6, 17)):
        h.set_option(name, good)
        assert h.get_option(name) == good
        _expect(pkg, "ERR_SHAPE", h.set_option, name, bad)
    _expect(pkg, "ERR_SHAPE", h.set_option, "no_such_option", 1)
    _expect(pkg, "ERR_DEVICE", h.profile, 1)
    h.close()


def test_missing_library_fails_loudly(monkeypatch, pkg):
    from paper_2605_02888_amd import binding
    monkeypatch.setattr(binding, "_lib", None)
    monkeypatch.setattr(binding, "LIB_PATH", os.path.join(ROOT, "no_such_dir", "libspeckv.so"))
    with pytest.raises(ImportError):
        binding.load_library()


def test_product_package_does_not_touch_the_oracle():
    # The HIP package must not import, load or link the oracle, and the oracle must not import it.
    for folder, banned in (("paper_2605_02888_amd", ("oracle", "speckv_oracle")), ("oracle", ("paper_2605_02888_amd", "libspeckv.so"))):
        for dirpath, _, files in os.walk(os.path.join(ROOT, folder)):
            if "_build" in dirpath or "__pycache__" in dirpath:
                continue
            for f in files:
                if not f.endswith((".py", ".cpp", ".hip", ".h", ".c")):
                    continue
                text = open(os.path.join(dirpath, f)).read()
                for word in banned:
                    assert word not in text, (os.path.join(dirpath, f), word)


def test_bench_refuses_more_than_one_gpu():
    # every box of this build has one GPU; sequences shard with no exchange, so N GPUs would be N copies
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode != 0 and "one GPU" in r.stderr and r.stdout.strip() == ""


def test_profile_summary_condenses_rocprofv3_csv(tmp_path, capsys):
    # the helper that turns rocprofv3's CSV files into the few lines kept under profiles/
    from paper_2605_02888_amd import profile_summary
    d = tmp_path / "trace" / "host" / "1234"
    d.mkdir(parents=True)
    (d / "c3_kernel_stats.csv").write_text(
        '"Name","Calls","TotalDurationNs","AverageNs","Percentage","MinNs","MaxNs","StdDev"\n'
        '"void speckv::row_stats_pair_kernel<2, 256, 2, false>(void const*, int)",10,1640000,164000.0,80.0,160000,170000,1.0\n'
        '"void at::native::vectorized_elementwise_kernel<4>(int)",5,5000,1000.0,0.1,900,1100,1.0\n')
    (d / "c3_counter_collection.csv").write_text(
        '"Dispatch_Id","Kernel_Name","Counter_Name","Counter_Value"\n'
        '1,"void speckv::probe_copy_kernel(uint4 const*, uint4*, long)","FETCH_SIZE",524300.0\n'
        '2,"void speckv::probe_copy_kernel(uint4 const*, uint4*, long)","FETCH_SIZE",524308.0\n'
        '3,"some_other_kernel(int)","FETCH_SIZE",1.0\n')
    assert profile_summary.main([str(tmp_path)]) == 0
    out = capsys.readouterr().out
    assert "row_stats_pair_kernel<2, 256, 2, false>" in out and "164.00" in out and "1.640" in out
    assert "vectorized_elementwise" not in out and "some_other_kernel" not in out
    line = [l for l in out.splitlines() if l.startswith("probe_copy_kernel")][0].split()
    assert line[1:] == ["FETCH_SIZE", "2", "524304.0", "524300.0", "524308.0"]
    assert profile_summary.main([]) == 2


def test_traffic_figures_are_tied_to_the_sources_they_were_measured_on():
    # bench.py reports roofline.traffic from profiles/ only while the digest recorded there is that
    # of the library's current sources
    import sys
    sys.path.insert(0, ROOT)
    import bench
    digest = bench.kernel_sources_digest()
    assert re.fullmatch(r"[0-9a-f]{16}", digest) and digest == bench.kernel_sources_digest()
    path = os.path.join(ROOT, "profiles", "row_stats_c3_traffic.txt")
    vals = dict(l.split()[:2] for l in open(path) if l.strip() and not l.startswith("#"))
    assert re.fullmatch(r"[0-9a-f]{16}", vals["kernel_sources_digest"])
    alg = {"row_stats_pair_bytes_per_launch": 1116340224, "row_stats_target_bytes_per_launch": 591003648,
           "row_stats_draft_bytes_per_launch": 525336576}
    for k, nbytes in alg.items():   # measured traffic: at least the algorithmic bytes, and within 1 % of them
        assert nbytes <= int(vals[k]) <= nbytes * 1.01, k
