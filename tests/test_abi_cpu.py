"""No-GPU checks of the boundary: the library loads, exports every symbol the header
declares, and its host-only entry points behave as documented."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "hot.h")


@pytest.fixture(scope="module")
def hot():
    from paper_2604_04736_amd import binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2604_04736_amd import build
        build.build_libhot()
    return binding


def _declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hot_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported(hot):
    names = _declared_symbols()
    assert set(names) == set(hot.EXPORTS), names
    L = hot.lib()
    for name in names:
        assert getattr(L, name) is not None


def _declared_return_types():
    """{name: C return type} for every function include/hot.h declares."""
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    out = {}
    for m in re.finditer(r"^\s*((?:const\s+)?[A-Za-z_0-9]+(?:\s*\*)?)\s*\b(hot_[a-z_]+)\s*\(", text, re.M):
        out[m.group(2)] = re.sub(r"\s+", " ", m.group(1)).replace(" *", "*").strip()
    return out


def test_binding_return_types_match_the_header(hot):
    """The ctypes restype of every entry point is the header's return type: a 64-bit byte count read as a
    32-bit int would be cut off (and turn negative) from 2 GiB on."""
    want = {"int": ctypes.c_int, "int64_t": ctypes.c_int64, "const char*": ctypes.c_char_p}
    declared = _declared_return_types()
    assert set(declared) == set(hot.EXPORTS)
    L = hot.lib()
    for name, ctype in declared.items():
        assert getattr(L, name).restype is want[ctype], (name, ctype, getattr(L, name).restype)
    assert {n for n, t in declared.items() if t != "int"} == set(hot.RESTYPES)


def test_workspace_query_over_many_shapes_is_consistent(hot):
    """Host arithmetic only: the answer is never negative for a valid layer, a multiple of 16 bytes, and
    covers at least two parts of what is split when it is not zero.  (With the present launch rules the
    largest answer is below 2 GiB; the return type is 64-bit all the same and is checked above.)"""
    import random
    r = random.Random(7)
    biggest = 0
    for _ in range(3000):
        rows = r.choice([1, 64, 255, 256, 1000, 7260, 16640, 65536, 1 << 20])
        k = 4 * r.randint(1, 4096)
        o = r.randint(1, 16384)
        s = r.choice([1, 2, 4, 16])
        b = hot.hot_linear_backward_workspace_bytes(rows, k, o, s)
        assert b >= 0 and b % 16 == 0, (rows, k, o, s, b)
        if b:
            per_w = 2 * (o * k + (o + 3) // 4 * 4) * 4
            per_x = s * rows * k * 4
            assert b >= 2 * min(per_w, per_x), (rows, k, o, s, b)
        biggest = max(biggest, b)
    assert biggest > 0


def test_launch_shape_query_over_many_shapes_is_consistent(hot):
    """Host arithmetic only: the code names a shape the 256/512/1024-row kernel has, never for fewer than 65 rows (up to 128 only its shapes of four waves x 32 rows, below 512 only its four-wave shapes), and for the
    input gradients never where rows of dy cannot be read in quads."""
    import random
    r = random.Random(11)
    singles = {211, 221, 411, 421, 811, 821, 841, 1621}
    seen = set()
    for _ in range(4000):
        rows = r.choice([1, 64, 65, 100, 128, 129, 255, 256, 511, 512, 1000, 1530, 2048, 4096, 7260, 16640, 65536])
        k = 4 * r.randint(1, 2200)
        o = r.randint(1, 9000)
        s = r.choice([1, 2, 3, 4, 16])
        own = r.random() < 0.4
        f = hot.hot_linear_launch_shape(rows, k, o, s, 0, per_sample_x=own)
        g = hot.hot_linear_launch_shape(rows, k, o, s, 1, per_sample_x=own)
        if rows < 65:
            assert f == 0 and g == 0
        if rows < 129:
            assert f // 100 % 10 in (0, 2) and g // 100 in (0, 2), (rows, k, o, s, f, g)
        elif rows < 512:
            assert f // 100 % 10 in (0, 4) and g // 100 in (0, 4), (rows, k, o, s, f, g)
        if own or s == 1:
            assert f == 0 or f in singles, (rows, k, o, s, own, f)
        else:
            assert f == 0 or f in singles or (f % 1000 in (212, 412, 812, 822) and f // 1000 in ((0,) if s % 2 == 0 else (1, 2, 4))), (rows, k, o, s, f)
        assert g == 0 or (g in singles and o % 4 == 0), (rows, k, o, s, g)
        seen.update((f, g))
    assert {0, 221, 411, 421, 811, 821, 841, 1621, 212, 412, 812, 822} <= seen
    assert hot.hot_linear_launch_shape(7260, 540, 2160, 2, 0) == 822          # the SWIN layer of the benchmark
    with pytest.raises(hot.HotError):
        hot.hot_linear_launch_shape(7260, 540, 2160, 2, 3)


def test_one_pass_backward_shape_query_and_its_workspace(hot):
    """Host arithmetic only: the kernels that take both gradients in one pass are chosen up to 32 rows where a
    lane's registers hold the dx accumulators of all samples (16-row blocks x samples held <= 8), from 33 to 128
    rows (the waves split the rows) for one or two samples on layers of half a million weights; the workspace
    the call then asks for holds a whole number of dx blocks."""
    import random
    r = random.Random(5)
    seen = set()
    for _ in range(4000):
        rows = r.choice([1, 5, 16, 17, 32, 33, 50, 64, 65, 128, 129, 200])
        k = 4 * r.randint(1, 2200)
        o = r.randint(1, 9000)
        s = r.choice([1, 2, 3, 4, 5, 8, 9, 16])
        code = hot.hot_linear_launch_shape(rows, k, o, s, 2)
        want = hot.hot_linear_backward_workspace_bytes(rows, k, o, s)
        strips, tiles, block = (k + 63) // 64, (o + 15) // 16, s * rows * k * 4
        if rows > 32:
            eligible = rows <= 128 and s <= 2 and k * o >= 512 * 1024
            expect, budget = 100 + 10 * (2 if rows > 64 else 1) + 2, 768
        else:
            rb = 2 if rows > 16 else 1
            held = 2 if s <= 2 else (4 if s <= 4 else 8)
            eligible = s <= 8 and rb * held <= 8
            expect, budget = 10 * rb + held, (512 if rb * held <= 4 else 256)
        if not eligible:
            assert code == 0, (rows, k, o, s, code)
            continue
        if code == 0:        # not two parts (too few tiles, or too many strips for two rounds) and too few strips on their own
            assert strips < 200 and (tiles < 8 or budget // strips < 2), (rows, k, o, s)
            continue
        assert code == expect, (rows, k, o, s, code)
        assert want >= 2 * block or strips >= 200 or rows >= 128, (rows, k, o, s, want)
        seen.add(code)
    assert seen == {12, 14, 18, 22, 24, 112, 122}
    assert hot.hot_linear_launch_shape(16, 2160, 8640, 2, 2) == 12 and hot.hot_linear_launch_shape(64, 8192, 8192, 2, 2) == 112


def test_host_only_entry_points(hot):
    assert hot.hot_version() == 302
    assert hot.hot_strerror(0) == "success"
    assert "invalid" in hot.hot_strerror(hot.HOT_EINVAL)
    assert hot.hot_strerror(-99) == "unknown error code"
    assert hot.hot_recommended_ld(1) == 64
    assert hot.hot_recommended_ld(64) == 64
    assert hot.hot_recommended_ld(32_024) == 32_064
    assert hot.hot_recommended_ld(2_693_578) == 2_693_632
    assert hot.hot_recommended_ld(0) == hot.HOT_EINVAL


def test_struct_layout_matches_header(hot):
    # hot_desc: int64, int64, int32, int32, double, int32, uint32 -> 40 bytes, natural alignment
    assert ctypes.sizeof(hot.hot_desc) == 40
    assert hot.hot_desc.dataset_size.offset == 24 and hot.hot_desc.flags.offset == 36
    assert ctypes.sizeof(hot.hot_launch) == 16
    assert ctypes.sizeof(hot.hot_linear_desc) == 64 and hot.hot_linear_desc.s_local.offset == 48
    assert hot.hot_linear_desc.x_sample_stride.offset == 56
    assert ctypes.sizeof(hot.hot_adam) == 56 and hot.hot_adam.step.offset == 48
    assert ctypes.sizeof(hot.hot_rng) == 16 and hot.hot_rng.step.offset == 8 and hot.hot_rng.first_sample.offset == 12


def test_null_arguments_are_rejected_without_a_gpu(hot):
    L = hot.lib()
    assert L.hot_create(None, None) == hot.HOT_EINVAL
    assert L.hot_destroy(None) == hot.HOT_OK
    assert L.hot_forward(None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward(None, None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_kl(None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_static(None, None, None, None, None, None, None) == hot.HOT_EINVAL
    # beyond the capacity of the static scratch: refused before anything touches a GPU
    too_big = hot.hot_desc(hot.HOT_STATIC_MAX_WEIGHTS + 1, hot.HOT_STATIC_MAX_WEIGHTS + 1, 1, 1, 1.0, 0, 0)
    assert L.hot_forward_static(ctypes.byref(too_big), None, None, None, None, None, None) == hot.HOT_ERANGE
    assert "capacity" in hot.hot_strerror(hot.HOT_ERANGE)
    assert L.hot_set_launch(None, 0, None) == hot.HOT_EINVAL
    assert L.hot_get_launch(None, 0, None) == hot.HOT_EINVAL
    assert L.hot_last_hip_error(None) == 0
    assert L.hot_probe_copy(None, None, 16, 0, None) == hot.HOT_EINVAL
    assert L.hot_probe_streams(None, 16, 1, 1, None) == hot.HOT_EINVAL
    assert L.hot_stats_local(None, 1, 1, 1, None, None, None) == hot.HOT_EINVAL
    assert L.hot_stats_whole(None, 1, 1, 1, 0, None, None, None) == hot.HOT_EINVAL
    assert L.hot_stats_merge(None, None, None, 1, 1, 1, 0, None, None, None) == hot.HOT_EINVAL
    assert L.hot_linear_forward_rng(None, None, None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_linear_backward_rng(None, 1, 1.0, 0, *([None] * 13)) == hot.HOT_EINVAL
    assert L.hot_linear_backward_rng_ws(None, 1, 1.0, 0, *([None] * 12), None, 0, None) == hot.HOT_EINVAL
    assert L.hot_linear_backward_workspace_bytes(None) == hot.HOT_EINVAL
    # the workspace query is host arithmetic: a ViT layer at 16 640 rows wants parts, a small layer none
    per = 2 * (768 * 192 + 768) * 4
    assert hot.hot_linear_backward_workspace_bytes(16640, 192, 768, 2) in (2 * per, 4 * per, 8 * per, 16 * per)
    assert hot.hot_linear_backward_workspace_bytes(64, 128, 128, 4) == 0
    assert hot.hot_linear_backward_workspace_bytes(4096, 4096, 4096, 2) == 0
    assert L.hot_adam_step(None, 1, None, None, None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_dropout_rng(None, None, 0.5, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward_dropout_rng(None, None, 0.5, None, None, None) == hot.HOT_EINVAL
    assert L.hot_forward_dropout_units_rng(None, None, 0.5, 4, 0, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward_dropout_units_rng(None, None, 0.5, 4, 0, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward_rows(None, None, None, None, None, None, 0, 1, 0, 1, None, None, None) == hot.HOT_EINVAL
    assert L.hot_adam_forward(*([None] * 15)) == hot.HOT_EINVAL
    assert L.hot_backward_adam(None, None, None, None, None, None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward_adam_forward(*([None] * 14)) == hot.HOT_EINVAL
    assert L.hot_forward_rng(None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_backward_rng(None, None, None, None, None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_sample_eps(None, None, None, None) == hot.HOT_EINVAL
    assert L.hot_sample_bits(None, None, None, None) == hot.HOT_EINVAL
    out = ctypes.c_void_p()
    for bad in [hot.hot_desc(0, 0, 1, 1, 1.0, 0, 0),        # N < 1
                hot.hot_desc(8, 7, 1, 1, 1.0, 0, 0),        # ld < N
                hot.hot_desc(8, 8, 0, 1, 1.0, 0, 0),        # S_loc < 1
                hot.hot_desc(8, 8, 3, 2, 1.0, 0, 0),        # S < S_loc
                hot.hot_desc(8, 8, 1, 1, 0.0, 0, 0),        # |D| <= 0
                hot.hot_desc(8, 8, 1, 1, float("nan"), 0, 0),
                hot.hot_desc(8, 8, 1, 1, float("inf"), 0, 0),
                hot.hot_desc(8, 8, 1, 1, 1.0, 0, 3)]:       # unknown flag
        assert L.hot_create(ctypes.byref(out), ctypes.byref(bad)) == hot.HOT_EINVAL
        assert not out.value


def test_binding_error_objects(hot):
    # every failing call surfaces as HotError with the code and the library's message
    with pytest.raises(hot.HotError) as e:
        hot._check_planless(hot.HOT_EINVAL, "hot_adam_step")
    assert e.value.code == hot.HOT_EINVAL and "hot_adam_step" in str(e.value) and "invalid" in str(e.value)
    hot._check_planless(hot.HOT_OK, "hot_adam_step")
    with pytest.raises(hot.HotError) as e:
        hot._check(hot.HOT_ENOMEM, "hot_forward")
    assert e.value.code == hot.HOT_ENOMEM and "memory" in str(e.value)


def test_device_code_has_no_packed_instructions(tmp_path):
    """The library is built with packed fp32 arithmetic switched off, and the one kernel version that made
    the compiler emit a packed move (v_pk_mov_b32, to rotate vectors read from LDS) returned sporadic wrong
    values on the MI355X: no v_pk_* instruction may appear in the gfx950 code of any source file."""
    from concurrent.futures import ThreadPoolExecutor
    import subprocess
    from paper_2604_04736_amd import build

    def packed(src):
        out = tmp_path / (os.path.basename(src) + ".s")
        cmd = [build.HIPCC] + build.FLAGS + ["-S", "--cuda-device-only", "-o", str(out), src]
        res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
        assert res.returncode == 0, res.stdout[-2000:]
        return [line.strip() for line in open(out) if re.match(r"\s+v_pk_", line)]

    with ThreadPoolExecutor(max_workers=len(build.SRCS)) as pool:
        found = dict(zip(build.SRCS, pool.map(packed, build.SRCS)))
    assert all(not v for v in found.values()), {k: v[:3] for k, v in found.items() if v}

    # Every kernel that uses the matrix cores ends its runs of matrix instructions with explicit wait states
    # (mfma_results_settle in linear.hip: the compiler once left them out behind a branch and an accumulator
    # register was read before the matrix pipeline had written it).
    kernels = 0
    for src in build.SRCS:
        text = open(tmp_path / (os.path.basename(src) + ".s")).read()
        for m in re.finditer(r"^(_Z\w+):[^\n]*\n(.*?)s_endpgm", text, re.S | re.M):
            if "v_mfma" in m.group(2):
                kernels += 1
                assert "s_nop 15" in m.group(2), m.group(1)
    assert kernels >= 10        # the instantiations of the kernels of the linear layer

    # The backward kernel of the largest workload (four chunks, two rows in flight, eps from its array) issues the 16
    # loads of a step of rows (2 rows x 4 chunks x (grad_w, eps)) ahead of the sums and then waits for the first.
    # With the narrow last tile's code unrolled beside the full tile's, the compiler once staggered them (a load, a
    # wait for it, the next load), which cost 2.5 % there.
    text = open(tmp_path / "backward.hip.s").read()
    name = r"_ZN\S*hot_backward_kernelILi4ELi2ELb1ELb1ELb0ENS_9StoreGradE\S*"
    body = re.search(r"^(%s):[^\n]*\n(.*?)s_endpgm" % name, text, re.S | re.M).group(2)
    shapes = []
    for block in re.split(r"^\.LBB\S+:", body, flags=re.M):
        ev = re.findall(r"(global_load_dwordx4|buffer_load_dwordx4)|s_waitcnt vmcnt\((\d+)\)", block)
        shapes.append("".join("L" if ld else "w%s " % n for ld, n in ev))
    assert any(re.search(r"L{16}w15 ", sh) for sh in shapes), [sh for sh in shapes if "LLLL" in sh]

    # ... and no kernel can read a result without them: the matrix builtins occur only inside MfmaAcc, whose
    # registers are private and handed out against an MfmaSettled alone, and only MfmaSettled's constructor
    # issues the wait states (so a read needs one constructed, i.e. the wait states issued).
    for src in build.SRCS:
        code = re.sub(r"//[^\n]*", "", open(src).read())
        calls = len(re.findall(r"__builtin_amdgcn_mfma_", code))
        if os.path.basename(src) != "linear.hip":
            assert calls == 0, src
            continue
        cls = re.search(r"class MfmaAcc \{(.*?)\n\};", code, re.S).group(1)
        assert calls == len(re.findall(r"__builtin_amdgcn_mfma_", cls)) == 3      # 16x16x4 f32, 32x32x2 f32, 32x32x16 bf16
        assert re.search(r"\n    V v_;\n\npublic:", "\n" + cls) and "read(const MfmaSettled &) const { return v_; }" in cls
        assert len(re.findall(r"mfma_results_settle\(\)", code)) == 2      # its definition and MfmaSettled's constructor
        assert "MfmaSettled() { mfma_results_settle(); }" in code
        assert len(re.findall(r"const MfmaSettled settled;", code)) >= 7     # one per kernel
