"""AddressSanitizer + UndefinedBehaviorSanitizer builds of the CPU checker (oracle/lora_oracle.c) and of the host
logic of the library (argument checks, slot table, placement), each linked into a small driver under
tests/sanitize/ and run here: the run must end clean (exit status 0, nothing on stderr) and return what the
ordinary builds return."""
import os
import struct
import subprocess

import numpy as np
import pytest

import oracle
from conftest import GOLDEN, ROOT
from paper_2602_24044_amd import binding as B
from paper_2602_24044_amd import build as libbuild
from paper_2602_24044_amd import workloads as wl
from test_oracle_slots import parse_trace

SAN = os.path.join(ROOT, "tests", "sanitize")
ENV = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1",
           OMP_NUM_THREADS="4")


def run_clean(cmd, stdin=None):
    res = subprocess.run(cmd, input=stdin, capture_output=True, text=True, env=ENV, timeout=300)
    assert res.returncode == 0 and res.stderr == "", (res.returncode, res.stderr[-4000:])
    return res.stdout


# ---------------------------------------------------------------------------
# the CPU checker
# ---------------------------------------------------------------------------
@pytest.fixture(scope="module")
def oracle_exe(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san_oracle") / "oracle_driver")
    subprocess.run(["gcc", "-g", "-O1", "-fopenmp", "-fno-fast-math", "-ffp-contract=off", "-fsanitize=address,undefined",
                    "-fno-sanitize-recover=all", "-fno-omit-frame-pointer", os.path.join(ROOT, "oracle", "lora_oracle.c"),
                    os.path.join(SAN, "oracle_driver.c"), "-o", exe], check=True)
    return exe


def _case(seed, T, d_in, d_out, ranks, with_bias, n_samples):
    rng = np.random.default_rng(seed)
    bits = lambda *shape: wl.to_bf16_bits(rng.standard_normal(shape).astype(np.float32))
    x, W = bits(T, d_in), bits(d_out, d_in)
    ids = rng.integers(-1, len(ranks), size=T).astype(np.int32)
    adapters = {i: (r, 0.5 + i, bits(r, d_in) if r else None, bits(d_out, r) if r else None) for i, r in enumerate(ranks)}
    bias = bits(d_out) if with_bias else None
    ts = rng.integers(0, max(T, 1), size=n_samples if T else 0).astype(np.int32)
    ns = rng.integers(0, d_out, size=ts.shape[0]).astype(np.int32)
    return x, W, ids, adapters, bias, ts, ns


def _write_case(path, x, W, ids, adapters, bias, ts, ns):
    T, d_in = x.shape
    n = len(adapters)
    with open(path, "wb") as f:
        f.write(struct.pack("6i", T, d_in, W.shape[0], n, int(bias is not None), ts.shape[0]))
        f.write(x.tobytes() + W.tobytes() + ids.tobytes())
        f.write(np.array([adapters[i][0] for i in range(n)], dtype=np.int32).tobytes())
        f.write(np.array([float(np.float32(adapters[i][1])) for i in range(n)], dtype=np.float64).tobytes())
        for i in range(n):
            if adapters[i][0] > 0:
                f.write(adapters[i][2].tobytes() + adapters[i][3].tobytes())
        if bias is not None:
            f.write(bias.tobytes())
        f.write(ts.tobytes() + ns.tobytes())


@pytest.mark.parametrize("seed,T,d_in,d_out,ranks,with_bias,n_samples", [
    (0, 37, 24, 19, [8, 0, 16, 3], False, 50),     # ragged sizes, a rank-0 adapter, an odd rank, backbone-only tokens
    (1, 5, 7, 3, [1], True, 9),                    # bias, sizes below any vector width
    (2, 0, 8, 8, [8], False, 0),                   # empty batch
    (3, 12, 16, 8, [], True, 0),                   # no adapters at all, no samples
    (4, 64, 128, 96, [32, 64, 8, 16, 24], True, 200),
])
def test_checker_runs_clean_and_agrees_with_the_ordinary_build(oracle_exe, tmp_path, seed, T, d_in, d_out, ranks,
                                                               with_bias, n_samples):
    x, W, ids, adapters, bias, ts, ns = _case(seed, T, d_in, d_out, ranks, with_bias, n_samples)
    if not ranks:
        ids[:] = -1
    _write_case(tmp_path / "case.bin", x, W, ids, adapters, bias, ts, ns)
    run_clean([oracle_exe, str(tmp_path / "case.bin"), str(tmp_path / "out.bin")])
    raw = open(tmp_path / "out.bin", "rb").read()
    assert struct.unpack("2i", raw[:8]) == (0, 0)
    got = np.frombuffer(raw[8:], dtype=np.float64)
    y = got[:T * d_out].reshape(T, d_out)
    y_at = got[T * d_out:]
    assert np.array_equal(y, oracle.project(x, W, ids, adapters, bias=bias))
    assert np.array_equal(y_at, oracle.project_at(x, W, ids, adapters, ts, ns, bias=bias))


def test_checker_error_returns_run_clean(oracle_exe, tmp_path):
    x, W, ids, adapters, bias, ts, ns = _case(9, 6, 8, 8, [8], False, 4)
    ids[3] = 5            # names an adapter that does not exist
    ns[1] = 8             # a sample outside the output
    _write_case(tmp_path / "case.bin", x, W, ids, adapters, bias, ts, ns)
    run_clean([oracle_exe, str(tmp_path / "case.bin"), str(tmp_path / "out.bin")])
    raw = open(tmp_path / "out.bin", "rb").read()
    assert struct.unpack("2i", raw[:8]) == (-1, -2) and len(raw) == 8


# ---------------------------------------------------------------------------
# host logic of the library
# ---------------------------------------------------------------------------
@pytest.fixture(scope="module")
def host_exe(tmp_path_factory):
    return libbuild.build_sanitized(str(tmp_path_factory.mktemp("san_host")), os.path.join(SAN, "host_driver.cpp"))


def _load_line(in_use, reqs):
    return "load %d %s %d %s" % (len(in_use), " ".join(map(str, in_use)), len(reqs),
                                 " ".join("%d %d %d" % r for r in reqs))


def _expect_load(tab_state, result):
    """The two lines the driver prints for a load: result = [(slot, copied)] or a status code."""
    head = "load 0 " + " ".join("%d:%d" % (s, int(c)) for s, c in result) if isinstance(result, list) else f"load {result}"
    return [head.rstrip(), "state " + " ".join(map(str, tab_state))]


def test_slot_table_hand_trace_and_random_sequences(host_exe):
    script, want = [], []
    n_slots, calls = parse_trace(os.path.join(GOLDEN, "slot_trace.txt"))
    script.append(f"ctx {n_slots} 32 63 1 1 64 64")
    want.append("ctx 0")
    for in_use, reqs, exp, state in calls:
        script.append(_load_line(in_use, reqs))
        want += _expect_load(state, B.LORA_ERR_SLOTS_EXHAUSTED if exp is None else exp)
    # random sequences against the slot oracle, with layers and several projections in the configuration
    rng = np.random.default_rng(7)
    n_slots, n_ids = 6, 20
    script.append(f"ctx {n_slots} 32 {n_ids - 1} 3 2 64 64 128 24")
    want.append("ctx 0")
    tab = oracle.SlotTable(n_slots)
    for _ in range(400):
        ads = rng.choice(n_ids, size=int(rng.integers(1, 4)), replace=False)
        reqs = [(int(a), int(rng.choice([0, 8, 16, 32])), int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1)
                for a in ads]
        in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 7)), replace=False)]
        script.append(_load_line(in_use, reqs))
        try:
            res = tab.load(reqs, in_use)
        except oracle.SlotsExhausted:
            res = B.LORA_ERR_SLOTS_EXHAUSTED
        want += _expect_load(tab.adapter, res)
        script.append(f"map {n_ids}")
        want.append("map " + " ".join(map(str, tab.id2slot(n_ids).tolist())))
    out = run_clean([host_exe], stdin="\n".join(script) + "\n").splitlines()
    assert out == want


def test_paged_slot_table_hand_trace_and_random_sequences(host_exe):
    script, want = [], []
    n_slots, n_pages, calls = parse_trace(os.path.join(GOLDEN, "page_trace.txt"))
    script.append(f"ctxp {n_slots} 32 63 1 {n_pages} 1 64 64")
    want.append("ctx 0")
    for in_use, reqs, exp, state, pages in calls:
        script += [_load_line(in_use, reqs), "pages"]
        want += _expect_load(state, B.LORA_ERR_SLOTS_EXHAUSTED if exp is None else exp)
        want.append("pages " + " ".join(map(str, pages)))
    rng = np.random.default_rng(11)
    n_slots, n_ids, n_pages = 6, 20, 9
    script.append(f"ctxp {n_slots} 32 {n_ids - 1} 2 {n_pages} 2 64 64 128 24")
    want.append("ctx 0")
    tab = oracle.PagedSlotTable(n_slots, n_pages)
    for _ in range(400):
        ads = rng.choice(n_ids, size=int(rng.integers(1, 4)), replace=False)
        reqs = [(int(a), int(rng.choice([0, 8, 16, 32])), int(rng.integers(0, n_slots)) if rng.random() < 0.1 else -1)
                for a in ads]
        in_use = [int(v) for v in rng.choice(n_ids, size=int(rng.integers(0, 7)), replace=False)]
        script += [_load_line(in_use, reqs), "pages"]
        try:
            res = tab.load(reqs, in_use)
        except oracle.SlotsExhausted:
            res = B.LORA_ERR_SLOTS_EXHAUSTED
        want += _expect_load(tab.adapter, res)
        want.append("pages " + " ".join(map(str, tab.first_page)))
    out = run_clean([host_exe], stdin="\n".join(script) + "\n").splitlines()
    assert out == want


def test_argument_errors_and_queries(host_exe):
    script = ["ctx 2 16 7 1 1 64 64",
              "load 0 1 9 8 -1", "load 0 1 1 32 -1", "load 0 1 1 12 -1", "load 0 1 1 8 2", "load 0 1 1 -8 -1",
              "load 1 99 1 1 8 -1", "load 0 0", "bucket",
              "ctx 0 16 7 1 1 64 64", "ctx 2 12 7 1 1 64 64", "ctx 2 16 7 1 1 60 64", "ctx 2 16 7 1 0", "ctx 2 16 7 300 1 64 64",
              "slab 32 32 256 1 2 64 64 4096 14336", "slab 32 32 256 4 2 64 64 4096 14336", "slab 0 32 256 1 1 64 64"]
    script += [f"str {s}" for s in range(-1, 14)]
    out = run_clean([host_exe], stdin="\n".join(script) + "\n").splitlines()
    empty = "state -1 -1"
    want = ["ctx 0"]
    for st in (B.LORA_ERR_ID_RANGE, B.LORA_ERR_RANK_EXCEEDS_SMAX, B.LORA_ERR_SHAPE, B.LORA_ERR_SLOT_RANGE,
               B.LORA_ERR_INVALID_ARG, B.LORA_ERR_ID_RANGE):
        want += [f"load {st}", empty]
    want += ["load 0", empty, f"bucket {B.LORA_ERR_HIP}"]
    assert out[:len(want)] == want
    rest = out[len(want):]
    assert all(line.split()[1] != "0" for line in rest[:5]), rest[:5]      # every bad configuration is refused
    proj = [(64, 64), (4096, 14336)]
    assert rest[5] == "slab %d" % B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 63))
    assert rest[6] == "slab %d" % B.lora_slab_bytes(B.make_config(proj, 32, 32, 256, 63, n_layers=4))
    assert rest[7] == "slab 0"
    assert rest[8:] == ["str " + B.lora_status_string(s) for s in range(-1, 14)]


def _law(cap):
    def thr(sizes, rates, a_max):
        total = 0.0
        for r in rates:
            total += r
        return min(total, cap) - a_max / 1024.0

    def starves(sizes, rates, a_max):
        load = 0.0
        for s, r in zip(sizes, rates):
            load += r * s
        return load > 8.0 * cap or len(sizes) > a_max
    return thr, starves


@pytest.mark.parametrize("seed,n,n_gpus,cap", [(0, 0, 2, 4.0), (1, 5, 1, 50.0), (2, 300, 6, 40.0), (3, 900, 4, 120.0),
                                                (4, 700, 2, 5.0), (5, 64, 0, 10.0)])
def test_placement_matches_the_ordinary_build(host_exe, seed, n, n_gpus, cap):
    rng = np.random.default_rng(seed)
    size = [int(v) for v in rng.choice([8, 16, 32], size=n)]
    rate = [float(v) for v in rng.choice([1.6, 0.8, 0.4, 0.1, 0.05, 0.025], size=n)]
    pairs = " ".join(f"{s} {r!r}" for s, r in zip(size, rate))
    out = run_clean([host_exe], stdin=f"prio {n} {pairs}\nplace {n_gpus} {cap!r} {n} {pairs}\n").splitlines()
    assert out[0] == ("prio 0 " + " ".join(map(str, B.lora_priority_sorting(size, rate)))).rstrip()
    try:
        gpu_of, a_max = B.lora_place_adapters(size, rate, n_gpus, *_law(cap))
        want = "place 0 " + " ".join(map(str, gpu_of)) + (" | " if gpu_of else "| ") + " ".join(map(str, a_max))
    except B.LoraError as e:
        want = f"place {e.status}"
    assert out[1].split() == want.split()
