"""Host-side logic of libadama that needs no GPU: the library loads, exports every symbol the
header declares, rejects bad arguments before touching the device, treats empty inputs as no-ops,
and its launch geometry covers every element of every tensor exactly once with in-bounds,
aligned accesses."""
import os
import re

import numpy as np
import pytest

from paper_2305_19982_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
FAKE = 0x7F0000000000          # a device-looking address; never dereferenced on these paths


@pytest.fixture(scope="module")
def lib():
    return binding.load()


def test_header_symbols_are_exported(lib):
    import glob

    names = set()
    for path in glob.glob(os.path.join(ROOT, "include", "*.h")):
        text = re.sub(r"/\*.*?\*/", "", open(path).read(), flags=re.S)
        names |= set(re.findall(r"\b(adama_[a-z_]+)\s*\(", text))
    assert {"adama_begin_step", "adama_fold", "adama_fold_multi", "adama_apply", "adama_last_error",
            "adama_fold_opt_multi", "adama_apply_opt_multi", "adama_sgdm_fold_multi"} <= names
    assert len(names) >= 26
    for name in sorted(names):
        assert hasattr(lib, name), f"{name} declared in include/*.h but not exported"


def test_header_constants_match_library(lib):
    text = open(os.path.join(ROOT, "include", "adama.h")).read()
    declared = int(re.search(r"#define ADAMA_MAX_TENSORS_PER_LAUNCH (\d+)", text).group(1))
    assert binding.adama_max_tensors_per_launch() == declared


def test_loaded_library_matches_the_sources_beside_it(lib):
    """The build id a library carries is a hash of its sources and flags; the binding refuses (or
    rebuilds) a binary whose id differs, so an edited kernel is never tested against an old build."""
    from paper_2305_19982_amd import build

    assert re.fullmatch(r"[0-9a-f]{16}", binding.adama_build_id())
    assert binding.adama_build_id() == build.library_id() == build.source_id()
    assert not build.stale()
    assert build.library_id(os.path.join(ROOT, "include", "adama.h")) is None      # a file without the marker


def test_empty_inputs_are_noops(lib):
    binding.adama_begin_step(None, None, 0, 0.9, 0.999)
    binding.adama_fold(None, None, None, "bf16", 0, 4, 0.9, 0.999)
    binding.adama_fold_multi([], 0, "f16", 4, 0.9, 0.999)
    binding.adama_fold_multi([(None, None, None, 0), (None, None, None, 0)], None, "f32", 1, 0.9, 0.999)
    binding.adama_apply(None, None, None, 0, 1e-3, 1e-8, 0.9, 0.999, 1)
    binding.adama_apply_multi([], 0, 1e-3, 1e-8, 0.9, 0.999, 1)
    binding.adama_begin_step_multi([], 0, 0.9, 0.999)


BAD_FOLD = [
    (dict(m=None), binding.ERR_INVALID_ARG, "m is NULL"),
    (dict(v=None), binding.ERR_INVALID_ARG, "v is NULL"),
    (dict(grad=None), binding.ERR_INVALID_ARG, "grad is NULL"),
    (dict(N=0), binding.ERR_INVALID_ARG, "micro-batches"),
    (dict(N=-3), binding.ERR_INVALID_ARG, "micro-batches"),
    (dict(beta1=1.0), binding.ERR_INVALID_ARG, "[0, 1)"),
    (dict(beta2=-0.1), binding.ERR_INVALID_ARG, "[0, 1)"),
    (dict(beta2=float("nan")), binding.ERR_INVALID_ARG, "[0, 1)"),
    (dict(gdt=7), binding.ERR_UNSUPPORTED_DTYPE, "dtype"),
    (dict(m=FAKE + 2), binding.ERR_INVALID_ARG, "not aligned"),
    (dict(grad=FAKE + 1, gdt=binding.BF16), binding.ERR_INVALID_ARG, "not aligned"),
    (dict(grad=FAKE + 2, gdt=binding.F32), binding.ERR_INVALID_ARG, "not aligned"),
    (dict(n=(1 << 40) + 1), binding.ERR_TOO_LARGE, "ADAMA_MAX_ELEMS"),
]


@pytest.mark.parametrize("override,status,text", BAD_FOLD, ids=[str(b[0]) for b in BAD_FOLD])
def test_fold_rejects_bad_arguments(lib, override, status, text):
    args = dict(m=FAKE, v=FAKE + (1 << 30), grad=FAKE + (2 << 30), gdt=binding.BF16, n=1000, N=4, beta1=0.9,
                beta2=0.999)
    args.update(override)
    with pytest.raises(binding.AdamaError) as ei:
        binding.adama_fold(args["m"], args["v"], args["grad"], args["gdt"], args["n"], args["N"], args["beta1"],
                           args["beta2"])
    assert ei.value.status == status
    assert text in ei.value.message
    assert text in binding.adama_last_error()
    with pytest.raises(binding.AdamaError) as ei2:
        binding.adama_fold_multi([(FAKE, FAKE + 4096, FAKE + 8192, 16), (args["m"], args["v"], args["grad"], args["n"])],
                                 None, args["gdt"], args["N"], args["beta1"], args["beta2"])
    assert ei2.value.status == status
    if "NULL" in text or "aligned" in text or "MAX_ELEMS" in text:
        assert "tensor 1" in ei2.value.message


def test_fold_multi_rejects_null_list_and_negative_count(lib):
    st = lib.adama_fold_multi(None, 3, binding.F32, 1, 0.9, 0.999, None)
    assert st == binding.ERR_INVALID_ARG and "list is NULL" in binding.adama_last_error()
    lst = binding.tensor_list([(FAKE, FAKE, FAKE, 4)])
    st = lib.adama_fold_multi(lst, -1, binding.F32, 1, 0.9, 0.999, None)
    assert st == binding.ERR_INVALID_ARG and "negative" in binding.adama_last_error()


BAD_APPLY = [
    (dict(t=0), "t >= 1"),
    (dict(t=-5), "t >= 1"),
    (dict(theta=None), "theta is NULL"),
    (dict(m=None), "m is NULL"),
    (dict(lr=float("inf")), "lr"),
    (dict(eps=-1e-8), "eps"),
    (dict(eps=float("nan")), "eps"),
    (dict(beta1=1.0), "[0, 1)"),
    (dict(beta2=1.5), "[0, 1)"),
]


@pytest.mark.parametrize("override,text", BAD_APPLY, ids=[str(b[0]) for b in BAD_APPLY])
def test_apply_rejects_bad_arguments(lib, override, text):
    args = dict(theta=FAKE, m=FAKE + (1 << 30), v=FAKE + (2 << 30), n=100, lr=1e-3, eps=1e-8, beta1=0.9, beta2=0.999, t=1)
    args.update(override)
    with pytest.raises(binding.AdamaError) as ei:
        binding.adama_apply(args["theta"], args["m"], args["v"], args["n"], args["lr"], args["eps"], args["beta1"],
                            args["beta2"], args["t"])
    assert ei.value.status == binding.ERR_INVALID_ARG and text in ei.value.message


def test_fused_entry_points_validate_like_their_parts(lib):
    ok = dict(theta=FAKE, m=FAKE + (1 << 30), v=FAKE + (2 << 30), grad=FAKE + (3 << 30))
    binding.adama_fold_first(None, None, None, "bf16", 0, 4, 0.9, 0.999)
    binding.adama_fold_last_apply(None, None, None, None, "f16", 0, 4, 1e-3, 1e-8, 0.9, 0.999, 1)
    binding.adama_fold_first_multi([], 0, "f32", 2, 0.9, 0.999)
    binding.adama_fold_last_apply_multi([], 0, "f32", 2, 1e-3, 1e-8, 0.9, 0.999, 5)
    for bad, text in ((dict(N=0), "micro-batches"), (dict(beta1=1.0), "[0, 1)"), (dict(m=None), "m is NULL"),
                      (dict(gdt=9), "dtype")):
        a = dict(ok, gdt=binding.BF16, N=4, beta1=0.9, beta2=0.999)
        a.update(bad)
        with pytest.raises(binding.AdamaError) as ei:
            binding.adama_fold_first(a["m"], a["v"], a["grad"], a["gdt"], 100, a["N"], a["beta1"], a["beta2"])
        assert text in ei.value.message
    for bad, text in ((dict(t=0), "t >= 1"), (dict(theta=None), "theta is NULL"), (dict(grad=None), "grad is NULL"),
                      (dict(eps=-1.0), "eps"), (dict(N=-1), "micro-batches"), (dict(lr=float("nan")), "lr")):
        a = dict(ok, gdt=binding.F32, N=4, beta1=0.9, beta2=0.999, lr=1e-3, eps=1e-8, t=1)
        a.update(bad)
        with pytest.raises(binding.AdamaError) as ei:
            binding.adama_fold_last_apply(a["theta"], a["m"], a["v"], a["grad"], a["gdt"], 100, a["N"], a["lr"],
                                          a["eps"], a["beta1"], a["beta2"], a["t"])
        assert ei.value.status in (binding.ERR_INVALID_ARG,) and text in ei.value.message


def test_rescale_apply_validation(lib):
    binding.adama_rescale_apply(None, None, None, 0, 0.5, 0.25, 1e-3, 1e-8, 0.9, 0.999, 1)
    for bad, text in ((dict(m_scale=-1.0), "m_scale"), (dict(v_scale=float("inf")), "v_scale"), (dict(t=0), "t >= 1"),
                      (dict(theta=None), "theta is NULL")):
        a = dict(theta=FAKE, m=FAKE + (1 << 30), v=FAKE + (2 << 30), m_scale=0.5, v_scale=0.25, t=1)
        a.update(bad)
        with pytest.raises(binding.AdamaError) as ei:
            binding.adama_rescale_apply(a["theta"], a["m"], a["v"], 100, a["m_scale"], a["v_scale"], 1e-3, 1e-8, 0.9,
                                        0.999, a["t"])
        assert text in ei.value.message


def test_option_validation(lib):
    """The *_opt calls: NULL options are accepted, bad ones are rejected before anything is queued."""
    fold = [(FAKE, FAKE + (1 << 30), FAKE + (2 << 30), 100)]
    upd = [(FAKE + (3 << 30), FAKE, FAKE + (1 << 30), FAKE + (2 << 30), 100)]
    st = [(FAKE + (3 << 30), FAKE, FAKE + (1 << 30), 100)]
    binding.adama_fold_opt_multi([], 0, "bf16", 4, 0.9, 0.999, None)
    binding.adama_fold_first_opt_multi([], 0, "bf16", 4, 0.9, 0.999, (0.0, 1.0 / 1024))
    binding.adama_fold_last_apply_opt_multi([], 0, "f16", 4, 1e-3, 1e-8, 0.9, 0.999, 1, binding.options(0.01, 0.5))
    binding.adama_apply_opt_multi([], 0, 1e-3, 1e-8, 0.9, 0.999, 1, (0.01, 1.0))
    binding.adama_rescale_apply_opt_multi([], 0, 0.5, 0.25, 1e-3, 1e-8, 0.9, 0.999, 1, (0.01, 1.0))
    for bad, text in (((-0.1, 1.0), "weight_decay"), ((float("nan"), 1.0), "weight_decay"), ((0.0, 0.0), "grad_scale"),
                      ((0.0, -2.0), "grad_scale"), ((0.0, float("inf")), "grad_scale")):
        for call in (lambda o: binding.adama_fold_opt_multi(fold, None, "bf16", 4, 0.9, 0.999, o),
                     lambda o: binding.adama_fold_first_opt_multi(fold, None, "bf16", 4, 0.9, 0.999, o),
                     lambda o: binding.adama_fold_last_apply_opt_multi(upd, None, "bf16", 4, 1e-3, 1e-8, 0.9, 0.999, 1, o),
                     lambda o: binding.adama_apply_opt_multi(st, None, 1e-3, 1e-8, 0.9, 0.999, 1, o),
                     lambda o: binding.adama_rescale_apply_opt_multi(st, None, 0.5, 0.25, 1e-3, 1e-8, 0.9, 0.999, 1, o),
                     lambda o: binding.adama_sgdm_fold_multi([(None, FAKE, FAKE + (1 << 30), 10)], None, "f32", 2, o),
                     lambda o: binding.adama_sgdm_apply_multi([(FAKE, FAKE + (1 << 30), None, 10)], None, 0.1, o)):
            with pytest.raises(binding.AdamaError) as ei:
                call(bad)
            assert ei.value.status == binding.ERR_INVALID_ARG and text in ei.value.message
    # the other checks of the plain calls still apply
    with pytest.raises(binding.AdamaError) as ei:
        binding.adama_fold_opt_multi(fold, None, "bf16", 0, 0.9, 0.999, None)
    assert "micro-batches" in ei.value.message
    with pytest.raises(binding.AdamaError) as ei:
        binding.adama_apply_opt_multi(st, None, 1e-3, 1e-8, 0.9, 0.999, 0, (0.1, 1.0))
    assert "t >= 1" in ei.value.message


def test_sgdm_validation(lib):
    binding.adama_sgdm_begin_step_multi([], 0, 0.9)
    binding.adama_sgdm_fold_multi([(None, None, None, 0)], None, "bf16", 4)
    binding.adama_sgdm_fold_first_multi([], 0, "f16", 4, 0.9)
    binding.adama_sgdm_apply_multi([], 0, 0.1)
    binding.adama_sgdm_fold_last_apply_multi([], 0, "f32", 4, 0.1, (0.01, 0.5))
    th, b, g = FAKE, FAKE + (1 << 30), FAKE + (2 << 30)
    cases = [
        (lambda: binding.adama_sgdm_begin_step_multi([(None, None, None, 8)], None, 0.9), "b is NULL"),
        (lambda: binding.adama_sgdm_begin_step_multi([(None, b, None, 8)], None, -0.9), "momentum"),
        (lambda: binding.adama_sgdm_begin_step_multi([(None, b, None, 8)], None, float("nan")), "momentum"),
        (lambda: binding.adama_sgdm_fold_multi([(None, b, None, 8)], None, "bf16", 4), "grad is NULL"),
        (lambda: binding.adama_sgdm_fold_multi([(None, b, g + 1, 8)], None, "bf16", 4), "not aligned"),
        (lambda: binding.adama_sgdm_fold_multi([(None, b, g, 8)], None, "bf16", 0), "micro-batches"),
        (lambda: binding.adama_sgdm_fold_multi([(None, b, g, 8)], None, 5, 4), "dtype"),
        (lambda: binding.adama_sgdm_fold_first_multi([(None, b, g, 8)], None, "f32", 4, float("inf")), "momentum"),
        (lambda: binding.adama_sgdm_apply_multi([(None, b, None, 8)], None, 0.1), "theta is NULL"),
        (lambda: binding.adama_sgdm_apply_multi([(th, b, None, 8)], None, float("inf")), "lr"),
        (lambda: binding.adama_sgdm_fold_last_apply_multi([(th, b, None, 8)], None, "f16", 4, 0.1), "grad is NULL"),
        (lambda: binding.adama_sgdm_fold_last_apply_multi([(th, b, g, (1 << 40) + 1)], None, "f16", 4, 0.1), "MAX_ELEMS"),
    ]
    for call, text in cases:
        with pytest.raises(binding.AdamaError) as ei:
            call()
        assert text in ei.value.message, (text, ei.value.message)
    # an apply ignores the gradient field, a decay ignores theta and the gradient
    assert lib.adama_sgdm_begin_step_multi(binding.sgdm_list([(None, None, None, 0)]), 1, 0.9, None) == binding.OK


def test_begin_step_hyper_parameters(lib):
    with pytest.raises(binding.AdamaError):
        binding.adama_begin_step(FAKE, FAKE + 4096, 10, -0.5, 0.999)
    with pytest.raises(binding.AdamaError):
        binding.adama_begin_step(FAKE, FAKE + 4096, 10, 0.9, float("inf"))
    with pytest.raises(binding.AdamaError):
        binding.adama_begin_step(FAKE, None, 10, 0.9, 0.999)
    # beta2 above 1 is legal here (data-parallel decay by M*beta2) -- with n == 0 nothing is launched
    binding.adama_begin_step(None, None, 0, 0.9, 8 * 0.999)


# ---------------------------------------------------------------------------
# launch geometry
# ---------------------------------------------------------------------------
def _walk_and_check(entries, op, gdt):
    touched, nvec, nsc, launches = binding.adama_debug_walk(entries, op, gdt)
    for k, (tch, e) in enumerate(zip(touched, entries)):
        arr = np.frombuffer(tch, dtype=np.uint8)
        assert arr.size == e[4]
        assert np.all(arr == 1), f"tensor {k}: elements touched {np.unique(arr)} times"
    assert nvec * 4 + nsc == sum(e[4] for e in entries)
    return nvec, nsc, launches


@pytest.mark.parametrize("gdt,gb", [("f32", 4), ("bf16", 2), ("f16", 2)])
def test_geometry_aligned_tensors_use_vector_accesses(lib, gdt, gb):
    rng = np.random.default_rng(1)
    sizes = [0, 1, 3, 4, 5, 1023, 1024, 1025, 4095, 4096, 4097, 12345, 65536, 0, 100001]
    entries = []
    a = FAKE
    for n in sizes:
        entries.append((a + (3 << 32), a, a + (1 << 32), a + (2 << 32), n))
        a += (4 * n + 255) // 256 * 256
    nvec, nsc, launches = _walk_and_check(entries, 1, gdt)
    assert launches == 1
    assert nsc == sum(n % 4 for n in sizes)          # only the ragged tails go element by element
    del rng


@pytest.mark.parametrize("op,gdt,gb", [(0, "f32", 4), (1, "f32", 4), (1, "bf16", 2), (1, "f16", 2), (2, "f32", 4),
                                       (3, "bf16", 2), (3, "f32", 4), (4, "f16", 2), (4, "f32", 4), (5, "f32", 4),
                                       (6, "f32", 4), (7, "bf16", 2), (7, "f32", 4), (8, "f32", 4), (9, "f16", 2),
                                       (10, "bf16", 2), (10, "f32", 4)])
def test_geometry_misaligned_and_large(lib, op, gdt, gb):
    rng = np.random.default_rng(2)
    entries = []
    for i in range(40):
        n = int(rng.integers(1, 30000))
        pre = int(rng.integers(0, 4))
        co = bool(rng.integers(0, 2))
        a = FAKE + (i << 24) + 4 * pre
        b = FAKE + (1 << 36) + (i << 24) + 4 * (pre if co else (pre + 1) % 4)
        c = FAKE + (2 << 36) + (i << 24) + gb * pre
        th = FAKE + (6 << 36) + (i << 24) + 4 * (pre if (co or i % 3) else (pre + 2) % 4)
        entries.append((th, a, b, c, n))
    # one launch big enough for the larger chunks of long launches, with every misalignment
    for pre in range(4):
        n = (1 << 22) + 3 * pre + 1
        entries.append((FAKE + (7 << 36) + (pre << 28) + 4 * pre, FAKE + (3 << 36) + (pre << 28) + 4 * pre,
                        FAKE + (4 << 36) + (pre << 28) + 4 * pre, FAKE + (5 << 36) + (pre << 28) + gb * pre, n))
    nvec, nsc, launches = _walk_and_check(entries, op, gdt)
    assert launches == 1 and nvec > 0 and nsc > 0


def test_geometry_chunk_size_follows_launch_size(lib):
    """Short launches use 1024-element chunks, long ones the op's own shape; the size classes change at 2^20 and
    2^26 elements, where the residency bound (reported by adama_residency, applied from 2^23 on) may change too."""
    sizes = {n: binding.adama_launch_chunk("fold", n) for n in (1, (1 << 20) - 1, 1 << 20, 30_740_800, 1 << 26, 1 << 30)}
    assert sizes[1] == sizes[(1 << 20) - 1] == 1024
    assert sizes[1 << 20] == sizes[30_740_800] and sizes[1 << 26] == sizes[1 << 30]
    assert binding.adama_residency("fold", (1 << 23) - 1) == 0 < binding.adama_residency("fold", 1 << 23)
    assert binding.adama_residency("fold", (1 << 26) - 1) == binding.adama_residency("fold", 1 << 23)
    assert binding.adama_residency("fold", 1 << 26) == binding.adama_residency("fold", 1 << 30) > 0
    assert binding.adama_launch_chunk(99, 5) == 0
    for op in range(11):
        for n in (5, 1 << 22, 1 << 28):
            t = binding.adama_tuning(op, n)
            assert t["block"] in (64, 128, 256) and 1 <= t["groups_per_thread"] <= 8
            assert binding.adama_launch_chunk(op, n) == t["block"] * 4 * t["groups_per_thread"]
            assert t["policy_bits"] & 7 == 7 and t["policy_bits"] < 16      # all streams non-temporal; bit 8 per op
    assert binding.adama_tuning(99, 5)["block"] == 0 and binding.adama_tuning(99, 5)["policy_bits"] == 0
    # one launch past the upper threshold, misaligned start: every element once, in bounds
    n = (3 << 25) + 5
    entries = [(FAKE + (3 << 40) + 12, FAKE + 12, FAKE + (1 << 40) + 12, FAKE + (2 << 40) + 6, n)]
    touched, nvec, nsc, launches = binding.adama_debug_walk(entries, 1, "bf16")
    arr = np.frombuffer(touched[0], dtype=np.uint8)
    assert arr.size == n and arr.min() == 1 and arr.max() == 1 and launches == 1
    assert nvec * 4 + nsc == n and nsc <= 6


def test_geometry_many_tensors_split_into_launches(lib):
    cap = binding.adama_max_tensors_per_launch()
    rng = np.random.default_rng(3)
    entries = []
    a = FAKE
    for i in range(2 * cap + 17):
        n = int(rng.integers(0, 3000))
        entries.append((a + (3 << 32), a, a + (1 << 32), a + (2 << 32), n))
        a += 4 * n                                   # packed back to back: all misalignments occur
    nvec, nsc, launches = _walk_and_check(entries, 1, "bf16")
    assert launches == 3
    nvec, nsc, launches = _walk_and_check(entries, 4, "bf16")
    assert launches == 3
    nvec, nsc, launches = _walk_and_check(entries, 10, "bf16")
    assert launches == 3


def test_geometry_walk_flags_nothing_on_workload_shapes(lib):
    """The tensor lists of the reduced benchmark workloads, as the harness lays them out (tight packing)."""
    from synth import configs

    for name in ("c1", "c3", "c4"):
        w = configs.reduced(name)
        off = 0
        for idx in w.layers:
            entries, goff = [], 0
            for ti in idx:
                n = w.tensors[ti].n
                entries.append((FAKE + (3 << 36) + 4 * off, FAKE + 4 * off, FAKE + (1 << 36) + 4 * off,
                                FAKE + (2 << 36) + w.grad_bytes * goff, n))
                off += n
                goff += n
            for op in (1, 3, 4, 7, 9, 10):
                _walk_and_check(entries, op, w.gdtype)


def test_geometry_randomised_lists(lib):
    """Seeded random tensor lists with adversarial lengths (around multiples of every chunk size, zero,
    tiny), random misalignments of every array and random co-alignment, for every op and gradient
    format, below and above the large-launch threshold: every element exactly once, in bounds, vector
    accesses aligned."""
    rng = np.random.default_rng(20240607)
    chunks = (512, 1024, 2048, 4096)
    gdts = (("f32", 4), ("bf16", 2), ("f16", 2))
    for trial in range(66):
        op = trial % 11
        gdt, gb = gdts[(trial // 11) % 3]
        big = trial % 2 == 0
        entries, total = [], 0
        count = int(rng.integers(1, 30))
        for i in range(count):
            kind = int(rng.integers(0, 5))
            if kind == 0:
                n = int(rng.integers(0, 6))
            elif kind == 1:
                n = int(rng.choice(chunks)) * int(rng.integers(1, 6)) + int(rng.integers(-3, 4))
            elif kind == 2:
                n = int(rng.integers(1, 40000))
            elif kind == 3:
                n = int(rng.choice(chunks)) - int(rng.integers(0, 4))
            else:
                n = int(rng.integers(100000, 400000)) if big else int(rng.integers(1, 3000))
            n = max(n, 0)
            pre = [int(rng.integers(0, 4)) for _ in range(4)]
            if rng.integers(0, 3) > 0:                # two thirds of the tensors co-aligned
                pre = [pre[0]] * 4
            base = FAKE + (i << 26)
            entries.append((base + (1 << 40) + 4 * pre[0], base + (2 << 40) + 4 * pre[1], base + (3 << 40) + 4 * pre[2],
                            base + (4 << 40) + gb * pre[3], n))
            total += n
        if big and total < (1 << 20):
            entries.append((FAKE + (5 << 40) + 4, FAKE + (6 << 40) + 4, FAKE + (7 << 40) + 4, FAKE + (8 << 40) + gb,
                            (1 << 20) + int(rng.integers(0, 5000))))
        touched, nvec, nsc, launches = binding.adama_debug_walk(entries, op, gdt)
        for k, (tch, e) in enumerate(zip(touched, entries)):
            arr = np.frombuffer(tch, dtype=np.uint8)
            assert arr.size == e[4] and np.all(arr == 1), f"trial {trial} op {op} {gdt} tensor {k} (n={e[4]})"
        assert nvec * 4 + nsc == sum(e[4] for e in entries)
        assert launches == 1
