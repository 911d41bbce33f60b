"""C-ABI checks that need no GPU: the library loads, exports every declared
symbol, and rejects bad arguments before touching the device."""
import ctypes as C
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def binding():
    lib_path = os.path.join(ROOT, "paper_2503_05530_amd", "csrc", "libproximity.so")
    if not os.path.exists(lib_path):
        from paper_2503_05530_amd.build import build_library
        build_library(verbose=False)
    import paper_2503_05530_amd.binding as b
    return b


def declared_functions():
    text = open(os.path.join(ROOT, "include", "proximity.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(proximity_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(binding):
    names = declared_functions()
    assert "proximity_create" in names and "proximity_search_batch" in names and "proximity_stats" in names
    for name in names:
        assert hasattr(binding.lib, name), f"{name} is declared in proximity.h but not exported"
    assert sorted(binding.EXPORTED) == names


def test_abi_version_and_struct_layout(binding):
    assert binding.proximity_abi_version() == 9
    assert C.sizeof(binding.ProximityConfig) == 72
    assert C.sizeof(binding.ProximityStats) == 128
    assert C.sizeof(binding.ProximityLaunch) == 20
    text = open(os.path.join(ROOT, "include", "proximity.h")).read()
    limits = {m.group(1): eval(m.group(2).replace("u", "")) for m in
              re.finditer(r"#define PROXIMITY_MAX_(\w+)\s+(\(?[0-9u <]+\)?)", text)}
    assert limits == {"K": binding.MAX_K, "DIM": binding.MAX_DIM, "BATCH": binding.MAX_BATCH,
                      "CAPACITY": binding.MAX_CAPACITY}
    metrics = re.search(r"PROXIMITY_METRIC_L2 = (\d), PROXIMITY_METRIC_IP = (\d), PROXIMITY_METRIC_COSINE = (\d)", text)
    assert [int(v) for v in metrics.groups()] == [binding.METRIC_L2, binding.METRIC_IP, binding.METRIC_COSINE]


def make_cfg(b, **kw):
    vals = dict(struct_size=C.sizeof(b.ProximityConfig), dim=768, corpus=None, n_docs=0, corpus_dtype=0,
                capacity=10, k=10, policy=0, max_batch=8, device=0, rerank_factor=1, lsh_bits=0, lsh_planes=None,
                metric=0, flags=0)
    vals.update(kw)
    return b.ProximityConfig(**vals)


@pytest.mark.parametrize("kw", [
    dict(struct_size=8), dict(dim=0), dict(dim=100), dict(dim=8192), dict(k=0), dict(k=1000),
    dict(max_batch=0), dict(max_batch=1 << 20), dict(capacity=(1 << 20) + 1), dict(n_docs=1 << 31),
    dict(n_docs=5, corpus=None), dict(corpus_dtype=7), dict(policy=2), dict(device=-1),
    dict(k=100, rerank_factor=3), dict(rerank_factor=1 << 31), dict(lsh_bits=17, lsh_planes=4096),
    dict(lsh_bits=4, lsh_planes=None), dict(lsh_bits=4, lsh_planes=4096, capacity=300),
    dict(lsh_bits=16, lsh_planes=4096, capacity=32), dict(metric=3), dict(flags=2),
    dict(n_docs=5, corpus=4096 + 4),
])
def test_create_rejects_bad_config_before_any_gpu_work(binding, kw):
    b = binding
    h = C.c_void_p(123)
    rc = b.lib.proximity_create(C.byref(make_cfg(b, **kw)), C.byref(h))
    assert rc == b.ERR_INVALID_ARG
    assert h.value is None
    assert b.last_error(None) != ""


def test_null_arguments(binding):
    b = binding
    h = C.c_void_p()
    assert b.lib.proximity_create(None, C.byref(h)) == b.ERR_INVALID_ARG
    assert b.lib.proximity_create(C.byref(make_cfg(b)), None) == b.ERR_INVALID_ARG
    assert b.lib.proximity_search_batch(None, None, 1, 10, 0.5, None, None, None, None) == b.ERR_INVALID_ARG
    assert b.lib.proximity_knn_batch(None, None, 1, 10, None, None, None) == b.ERR_INVALID_ARG
    assert b.lib.proximity_stats(None, None) == b.ERR_INVALID_ARG
    assert b.lib.proximity_clear(None) == b.ERR_INVALID_ARG
    assert b.lib.proximity_profile_start(None) == b.ERR_INVALID_ARG
    n = C.c_uint32(0)
    assert b.lib.proximity_cache_dump(None, None, None, None, C.byref(n)) == b.ERR_INVALID_ARG
    b.lib.proximity_destroy(None)  # must be a no-op


def test_static_search_rejects_bad_arguments_before_any_gpu_work(binding):
    """proximity_knn_static has a workspace of fixed size: sizes beyond it, and every other bad argument,
    are refused with a message before the device is touched."""
    b = binding
    call = lambda **kw: b.lib.proximity_knn_static(*[dict(dict(
        corpus=4096, n_docs=100, dim=768, dtype=0, metric=0, queries=8192, n=1, k=10, out_ids=4096, out_dists=None,
        device=0, stream=None), **kw)[name] for name in (
        "corpus", "n_docs", "dim", "dtype", "metric", "queries", "n", "k", "out_ids", "out_dists", "device", "stream")])
    text = open(os.path.join(ROOT, "include", "proximity.h")).read()
    limits = {m.group(1): eval(m.group(2).replace("u", "")) for m in
              re.finditer(r"#define PROXIMITY_STATIC_MAX_(\w+)\s+(\(?[0-9u <]+\)?)", text)}
    assert limits == {"DOCS": b.STATIC_MAX_DOCS, "QUERIES": b.STATIC_MAX_QUERIES}
    assert call(n_docs=b.STATIC_MAX_DOCS + 1) == b.ERR_INVALID_ARG
    assert "PROXIMITY_STATIC_MAX_DOCS" in b.last_error(None)
    assert call(n=b.STATIC_MAX_QUERIES + 1) == b.ERR_BATCH_TOO_LARGE
    assert "PROXIMITY_STATIC_MAX_QUERIES" in b.last_error(None)
    for kw in (dict(dim=0), dict(dim=100), dict(dim=8192), dict(k=0), dict(k=241), dict(dtype=2), dict(metric=3),
               dict(corpus=None), dict(queries=None), dict(out_ids=None), dict(corpus=4100), dict(queries=8200),
               dict(device=-1), dict(device=64)):
        assert call(**kw) == b.ERR_INVALID_ARG, kw
        assert b.last_error(None) != ""


def test_build_flag_keeps_packed_float32_instructions_out_of_device_code(tmp_path):
    """The library is compiled with a target-feature switch that stops the compiler from pairing float
    operations into packed-float32 instructions.  The switch is live: the same two-float kernel compiles to a
    packed instruction without it and to none with it."""
    import subprocess
    from paper_2503_05530_amd.build import NO_PACKED_FP32, HIPCC_FLAGS
    assert all(f in HIPCC_FLAGS for f in NO_PACKED_FP32)
    src = tmp_path / "two_floats.hip"
    src.write_text("#include <hip/hip_runtime.h>\n"
                   "__global__ void axpy2(const float2* __restrict__ x, float2* __restrict__ y, float a, int n) {\n"
                   "  int i = blockIdx.x * blockDim.x + threadIdx.x;\n"
                   "  if (i < n) { float2 v = x[i], w = y[i]; w.x = a * v.x + w.x; w.y = a * v.y + w.y; y[i] = w; }\n"
                   "}\n")
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    packed = re.compile(r"\bv_pk_(add|mul|fma)_f32\b")
    counts = {}
    for name, extra in (("with", NO_PACKED_FP32), ("without", [])):
        out = tmp_path / f"{name}.s"
        subprocess.run([hipcc, "-O3", "--offload-arch=gfx950", "--cuda-device-only", "-S", "-o", str(out), str(src),
                        *extra], check=True, capture_output=True)
        counts[name] = len(packed.findall(out.read_text()))
    assert counts["with"] == 0 and counts["without"] > 0, counts


def test_device_assembly_is_free_of_two_patterns_the_compiler_does_not_guard(tmp_path):
    """The register-resident scan writes its matrix instructions in assembly, where the compiler inserts no idle
    states for them: an ordinary vector instruction that writes a register must be at least two issue slots ahead
    of a matrix instruction that reads it (accumulators set to zero by moves that the compiler sinks down to the
    first use have given wrong scores for two rows in eight).  The device code of the library is compiled to
    assembly and every matrix instruction's two preceding slots are checked."""
    import subprocess
    from paper_2503_05530_amd.build import CSRC, NO_PACKED_FP32
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    out = tmp_path / "device.s"
    subprocess.run([hipcc, "-O3", "-std=c++17", "--offload-arch=gfx950", "--cuda-device-only", "-S", *NO_PACKED_FP32,
                    "-o", str(out), os.path.join(CSRC, "proximity.hip")], check=True, capture_output=True)

    def registers(token):
        m = re.match(r"v\[(\d+):(\d+)\]$", token)
        if m:
            return set(range(int(m.group(1)), int(m.group(2)) + 1))
        m = re.match(r"v(\d+)$", token)
        return {int(m.group(1))} if m else set()

    found, n_matrix, kernel, recent = [], 0, None, []      # recent: (registers written, issue slots, text)
    for line in out.read_text().splitlines():
        m = re.match(r"^(_Z\S+):", line)
        if m:
            kernel, recent = m.group(1), []
            continue
        text = line.strip()
        if not text or text[0] in ";." or text.endswith(":"):
            continue
        op = text.split()[0]
        args = [a.strip() for a in text[len(op):].split(",")]
        if op.startswith("v_mfma"):
            n_matrix += 1
            reads = registers(args[1]) | registers(args[2]) | registers(args[3])
            slots = 0
            for written, width, what in reversed(recent):
                if slots >= 2:
                    break
                if written & reads:
                    found.append((kernel, what, text))
                    break
                slots += width
            recent.append((set(), 1, text))
        elif op == "s_nop":
            recent.append((set(), int(args[0]) + 1, text))
        elif op.startswith("v_") and not op.startswith("v_cmp"):
            recent.append((registers(args[0]), 1, text))
        else:
            recent.append((set(), 1, text))
        recent = recent[-8:]
    assert n_matrix > 2000          # (the scan kernels are in there, unrolled)
    assert not found, found[:4]

    # A second pattern in the same assembly: a scalar load through a pointer that is not the kernel's argument
    # block, sitting in a stretch where the execution mask was narrowed and no branch skips it.  Scalar
    # instructions ignore the mask, so such a load is issued whatever the lanes decided -- and a pointer that the
    # source dereferences only "if it is not null" is then read at address zero (this faulted a GPU once: the
    # compiler turns `cond_per_lane && p ? *p : x` into exactly this when p is the same for all lanes).
    lines = [l.strip() for l in out.read_text().splitlines()]
    lines = [l for l in lines if l and l[0] not in ";."]
    unguarded = []
    for i, text in enumerate(lines):
        if not text.startswith("s_load_dword") or "s[0:1]" in text:
            continue
        before = lines[max(0, i - 6):i]
        narrowed = [j for j, b in enumerate(before) if "saveexec" in b or re.search(r"s_(and|xor|andn2)_b64 exec,", b)]
        if narrowed and not any("s_cbranch_exec" in b or b.endswith(":") for b in before[narrowed[-1]:]):
            unguarded.append((text, before[narrowed[-1]:]))
    assert not unguarded, unguarded[:3]


def test_score_error_bound_by_hand_and_against_float32_arithmetic(binding):
    """The bound behind the exactness check of the index search: its closed form worked by hand, and that
    float32 scores computed in several summation orders really stay within it of the float64 scores."""
    import numpy as np
    b = binding
    E = b.lib.proximity_score_error_bound
    u = 2.0 ** -24
    # dim 768: g = (3 * 768 + 16) u + 2^-17 = 2320 u + 128 u
    g = 2448 * u
    assert E(0, 768, 1.0, 1.0) == pytest.approx(g * 3.0, rel=1e-15)
    assert E(0, 768, 2.0, 0.5) == pytest.approx(g * (0.25 + 2.0), rel=1e-15)
    assert E(1, 768, 2.0, 0.5) == pytest.approx(g * 2.0, rel=1e-15)
    assert E(2, 768, 2.0, 123.0) == pytest.approx(g * 8.0, rel=1e-15)
    assert E(0, 32, 1.0, 1.0) == pytest.approx(240 * u * 3.0, rel=1e-15)
    for bad in ((3, 768, 1.0, 1.0), (0, 0, 1.0, 1.0), (0, 768, -1.0, 1.0), (0, 768, 1.0, float("nan"))):
        assert np.isnan(E(*bad))
    rng = np.random.default_rng(40)
    for dim in (32, 768, 4096):
        x = (rng.standard_normal((300, dim)) * rng.uniform(0.2, 4.0, (300, 1))).astype(np.float32)
        q = (rng.standard_normal(dim) * 1.7).astype(np.float32)
        x64, q64 = x.astype(np.float64), q.astype(np.float64)
        x_max, q_len = np.sqrt((x64 * x64).sum(1)).max(), np.sqrt((q64 * q64).sum())
        exact = {0: (x64 * x64).sum(1) - 2 * x64 @ q64, 1: -2 * x64 @ q64,
                 2: -2 * (x64 @ q64) / np.sqrt((x64 * x64).sum(1))}
        for order in ("forward", "reverse", "pairwise"):
            if order == "pairwise":
                dot = (x * q[None, :]).sum(1, dtype=np.float32)
                nrm = (x * x).sum(1, dtype=np.float32)
            else:
                cols = range(dim) if order == "forward" else range(dim - 1, -1, -1)
                dot, nrm = np.zeros(300, np.float32), np.zeros(300, np.float32)
                for c in cols:
                    dot = dot + x[:, c] * q[c]
                    nrm = nrm + x[:, c] * x[:, c]
            got = {0: nrm - np.float32(2) * dot, 1: np.float32(-2) * dot,
                   2: np.float32(-2) * dot * (np.float32(1) / np.sqrt(nrm))}
            for metric in (0, 1, 2):
                err = np.abs(got[metric].astype(np.float64) - exact[metric]).max()
                assert err <= E(metric, dim, q_len, x_max), (dim, order, metric, err)


def test_coarse_score_error_by_hand_and_against_rounded_operands(binding):
    """What a search that multiplies bfloat16 roundings may add to the score error: the closed form by hand, and
    scores formed in float32 from rounded queries against bfloat16 rows (a bfloat16 corpus) or against float32
    rows rounded the same way (a float32 corpus) really stay within the sum of both bounds of the float64 scores
    of the unrounded operands."""
    import numpy as np
    b = binding
    E, C1 = b.lib.proximity_score_error_bound, b.lib.proximity_coarse_score_error
    u = 2.0 ** -8 * 1.001
    assert C1(0, 1, 2.0, 0.5) == pytest.approx(u * 1.0, rel=1e-15)
    assert C1(1, 1, 2.0, 0.5) == pytest.approx(u * 1.0, rel=1e-15)
    assert C1(2, 1, 2.0, 123.0) == pytest.approx(u * 2.0, rel=1e-15)
    assert C1(0, 0, 2.0, 0.5) == pytest.approx(u * 2.002, rel=1e-15)
    assert C1(2, 0, 2.0, 123.0) == pytest.approx(u * 2.0 * 2.002, rel=1e-15)
    for bad in ((3, 1, 1.0, 1.0), (0, 2, 1.0, 1.0), (0, 1, -1.0, 1.0), (0, 0, 1.0, float("nan"))):
        assert np.isnan(C1(*bad))

    def to_bf16(v):          # round to nearest even, as float32 values
        bits = v.astype(np.float32).view(np.uint32).astype(np.uint64)
        bits = ((bits + 0x7fff + ((bits >> 16) & 1)) >> 16) << 16
        return bits.astype(np.uint32).view(np.float32)

    def off_grid(v):         # every element as far from its rounding as it gets, all to the same side
        return (to_bf16(v).astype(np.float64) * (1.0 + 2.0 ** -9 * 0.999)).astype(np.float32)

    rng = np.random.default_rng(41)
    worst = {0: 0.0, 1: 0.0}
    for corpus_dtype in (1, 0):
        for dim in ((256, 384) if corpus_dtype == 1 else (384, 768)):
            rows = (rng.standard_normal((400, dim)) * rng.uniform(0.2, 3.0, (400, 1))).astype(np.float32)
            for trial in range(6):
                q = (rng.standard_normal(dim) * rng.uniform(0.1, 5.0)).astype(np.float32)
                x = rows
                if trial == 5:
                    q, x = off_grid(q), off_grid(rows)
                if corpus_dtype == 1:
                    x = to_bf16(x)                           # the corpus itself
                x_mul, q_mul = to_bf16(x), to_bf16(q)        # what is multiplied
                x64, q64 = x.astype(np.float64), q.astype(np.float64)
                x_max, q_len = np.sqrt((x64 * x64).sum(1)).max(), np.sqrt((q64 * q64).sum())
                exact = {0: (x64 * x64).sum(1) - 2 * x64 @ q64, 1: -2 * x64 @ q64,
                         2: -2 * (x64 @ q64) / np.sqrt((x64 * x64).sum(1))}
                dot = (x_mul * q_mul[None, :]).sum(1, dtype=np.float32)
                nrm = (x * x).sum(1, dtype=np.float32)       # the rows' terms come from the rows as stored
                got = {0: nrm - np.float32(2) * dot, 1: np.float32(-2) * dot,
                       2: np.float32(-2) * dot * (np.float32(1) / np.sqrt(nrm))}
                for metric in (0, 1, 2):
                    err = np.abs(got[metric].astype(np.float64) - exact[metric]).max()
                    bound = E(metric, dim, q_len, x_max) + C1(metric, corpus_dtype, q_len, x_max)
                    assert err <= bound, (corpus_dtype, dim, trial, metric, err, bound)
                    worst[corpus_dtype] = max(worst[corpus_dtype], err / bound)
    assert worst[0] > 0.02 and worst[1] > 0.02     # (not vacuous: aligned roundings come within two orders of it)


def test_list_length_of_a_search_on_rounded_operands(binding):
    """The candidates such a search keeps: the closed form worked here from its definition, the values the header
    quotes, growth with k, with the corpus and with the dimension, and the float32 corpus (rows rounded too)
    asking for more than the bfloat16 one."""
    import math
    L = binding.lib.proximity_rounded_scan_list_length

    def by_hand(k, dtype, dim, n):
        delta = math.sqrt(dim) / 512 * (1.0 if dtype == 1 else 2.002)
        m = k * (math.exp(math.sqrt(2 * math.log(max(n / k, 2))) * delta) - 1)
        return k + math.ceil(m + 5 * math.sqrt(m) + 16)

    assert L(10, 0, 768, 1_000_000) == 46 and L(100, 1, 384, 8_000_000) == 159 and L(32, 0, 768, 24_000_000) == 97
    for k in (1, 10, 100, 240):
        for dtype in (0, 1):
            for dim in (256, 384, 768):
                for n in (1, 500, 1_000_000, 1 << 40):
                    assert L(k, dtype, dim, n) == by_hand(k, dtype, dim, n), (k, dtype, dim, n)
                    assert L(k, dtype, dim, n) >= k + 16
    assert L(10, 0, 768, 10**6) > L(10, 1, 768, 10**6) and L(10, 0, 768, 10**8) > L(10, 0, 768, 10**6)
    assert L(10, 0, 768, 10**6) > L(10, 0, 384, 10**6) and L(50, 0, 768, 10**6) > L(10, 0, 768, 10**6)
    for bad in ((0, 0, 768, 100), (241, 0, 768, 100), (10, 2, 768, 100), (10, 0, 0, 100), (10, 0, 5000, 100)):
        assert L(*bad) == 0


def probe_ranges(b, n, capacity, max_batch, listing, n_cu=256):
    import ctypes as C
    out = (C.c_uint32 * 200)()
    k = b.lib.proximity_probe_row_ranges(n, capacity, max_batch, listing, n_cu, out, 200)
    return list(out[:k])


def test_row_ranges_of_a_call_cover_it_in_order_within_the_score_buffers():
    """The host rule that cuts a large call into the row ranges probed beside the resolver (host arithmetic behind
    the C ABI): ranges are contiguous, in order, end on multiples of 64 (the resolver walks chunks of 64 rows),
    none is longer than the score buffers hold, and the last rows go in short ranges."""
    import paper_2503_05530_amd.binding as b
    budget = 512 << 20
    for capacity, max_batch in ((300, 8192), (10_000, 4096), (200_000, 4096), (1 << 20, 8192), (19_000, 8192)):
        ld = (capacity + max_batch + 63) // 64 * 64
        most = min(1536, max(64, budget // (2 * ld * 4) // 64 * 64))       # rows whose scores fit one buffer
        for listing in (0, 1):
            for n in list(range(1, 300, 7)) + list(range(most - 3, min(max_batch, most + 1500), 13)) + \
                    list(range(max(1, max_batch - 700), max_batch + 1, 11)):
                if n > max_batch:
                    continue
                ends = probe_ranges(b, n, capacity, max_batch, listing)
                assert ends and ends[-1] == n, (capacity, max_batch, listing, n, ends)
                starts = [0] + ends[:-1]
                for r0, r1 in zip(starts, ends):
                    assert 0 < r1 - r0 <= most and r0 % 64 == 0, (capacity, max_batch, listing, n, ends)
                if n <= most:
                    assert ends == [n]
                elif n - most > 1024:
                    assert ends[-1] - ends[-2] <= max(512, most // 2) + 64   # what remains after the last probe is short
    # the configuration of the probe microbenchmark: five ranges, the two last of 256 rows
    assert probe_ranges(b, 4096, 10_000, 4096, 1) == [1216, 2624, 3584, 3840, 4096]
    # bad arguments
    assert probe_ranges(b, 0, 10_000, 4096, 1) == [] and probe_ranges(b, 5000, 10_000, 4096, 1) == []
    assert probe_ranges(b, 64, 0, 4096, 1) == []
