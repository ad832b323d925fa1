"""The launch plan (chunk table + pointer table) is built on the host; check it
without a GPU through odsgd_plan_host: every element covered exactly once,
alignment rules, ordering, table contents.  Addresses are made up and never
dereferenced."""
import os

import pytest
from hypothesis import given, settings, strategies as st

from paper_2005_06728_amd import binding as B
from paper_2005_06728_amd import workloads as wl


def fake_layout(sizes, W, phases, base=0x7f0000000000):
    """Non-overlapping made-up addresses: role j gets its own 1 TiB region; inside it
    tensor k sits at a 1 KiB boundary plus phases[j] bytes."""
    def region(j):
        out, o = [], base + j * (1 << 40)
        for n in sizes:
            out.append(o + phases[j])
            o += ((4 * n + phases[j] + 1023) // 1024 + 1) * 1024
        return out
    w, v = region(0), region(1)
    g = [region(2 + m) for m in range(W)]
    u = [region(2 + W + m) for m in range(W)]
    return w, v, g, u


BLOCK = 65536  # bytes: two-half tiles live inside aligned blocks of this size


def rows_of_tensor(n):
    return 1 if n <= B.ROW_ELEMS else -(-n // B.ROW_ELEMS)


def check_plan(sizes, W, phases, pair_bit=15, layout=None):
    """Decode the plan for made-up addresses and check every structural rule.  Returns the chunks."""
    w, v, g, u = layout or fake_layout(sizes, W, phases)
    rows, chunks = B.odsgd_plan_host(sizes, w, v, g, u, W)
    K = len(sizes)
    # pointer table: one row per tensor, or per 2^29 elements of a larger one
    row_tensor, row_off = [], []
    for k in range(K):
        for j in range(rows_of_tensor(sizes[k])):
            row_tensor.append(k)
            row_off.append(j * B.ROW_ELEMS)
    assert len(rows) == len(row_tensor)
    for r, (k, o) in enumerate(zip(row_tensor, row_off)):
        want = [w[k], v[k]] + [g[m][k] for m in range(W)] + [u[m][k] for m in range(W)]
        if sizes[k] == 0:
            assert rows[r] == [0] * (4 + 3 * W)
            continue
        assert rows[r][:2 + 2 * W] == [p + 4 * o for p in want]
        assert rows[r][2 + 2 * W:] == [0] * (W + 2)
    # coverage: every element of every row exactly once; ordering: full chunks first
    per_row = {r: [] for r in range(len(rows))}
    seen_ragged = False
    for ch in chunks:
        r, vec, cnt, off, second = ch
        assert 0 <= r < len(rows) and 0 < cnt <= 256 and off < B.ROW_ELEMS + BLOCK // 4
        if second:
            assert vec and cnt == 256 and pair_bit and second == (1 << pair_bit) // 16 - 32
        for lo, hi in B.chunk_elements(ch):
            per_row[r].append((lo, hi, vec, bool(second)))
        if cnt < 256:
            seen_ragged = True
        else:
            assert not seen_ragged, "a full chunk after a ragged one"
    for r, (k, o) in enumerate(zip(row_tensor, row_off)):
        n = min(B.ROW_ELEMS, sizes[k] - o) if sizes[k] else 0
        pieces = sorted(per_row[r])
        pos = 0
        for lo, hi, vec, paired in pieces:
            assert lo == pos, "gap or overlap at element %d of row %d" % (pos, r)
            pos = hi
        assert pos == n
        all_ptrs = [w[k], v[k]] + [g[m][k] for m in range(W)] + [u[m][k] for m in range(W)]
        vec_ok = all(p % 16 == 0 for p in all_ptrs)
        same_tile = len({p % 1024 for p in all_ptrs}) == 1
        same_block = len({p % BLOCK for p in all_ptrs}) == 1
        base = w[k] + 4 * o
        for ch in chunks:
            if ch[0] != r:
                continue
            _, vec, cnt, off, second = ch
            assert vec == vec_ok
            start = base + 4 * off
            if second:
                # both halves inside one aligned block, the first in its lower half
                assert same_block and start % 512 == 0 and start % BLOCK < BLOCK // 2
            elif vec_ok and same_tile and cnt == 256:
                assert start % 1024 == 0, "full chunk does not start on a tile boundary"
        if vec_ok and same_block and pair_bit and n:
            # every aligned block that lies wholly inside the row is done with two-half tiles
            first_block = -(-base // BLOCK) * BLOCK
            nblocks = max(0, (base + 4 * n - first_block) // BLOCK)
            assert sum(1 for ch in chunks if ch[0] == r and ch[4]) == nblocks * (BLOCK // 1024)
        else:
            assert not any(ch[4] for ch in chunks if ch[0] == r)
    assert len(chunks) <= sum(-(-n // 256) + 2 * rows_of_tensor(n) for n in sizes if n)
    return chunks


@settings(max_examples=150, deadline=None)
@given(sizes=st.lists(st.one_of(st.integers(0, 40), st.integers(200, 1400), st.integers(4000, 9000),
                                st.integers(16000, 50000)),
                      min_size=1, max_size=7),
       W=st.integers(1, 5),
       phase_kind=st.sampled_from(["aligned", "same16", "same16far", "same4", "mixed16", "mixed4", "mixed1k"]),
       data=st.data())
def test_every_element_is_covered_exactly_once(sizes, W, phase_kind, data):
    roles = 2 + 2 * W
    if phase_kind == "aligned":
        phases = [0] * roles
    elif phase_kind == "same16":
        phases = [16 * data.draw(st.integers(1, 63))] * roles
    elif phase_kind == "same16far":
        phases = [16 * data.draw(st.integers(1, 4095))] * roles
    elif phase_kind == "mixed1k":
        phases = [1024 * data.draw(st.integers(0, 63)) for _ in range(roles)]
    elif phase_kind == "same4":
        phases = [4 * data.draw(st.integers(1, 255))] * roles
    elif phase_kind == "mixed16":
        phases = [16 * data.draw(st.integers(0, 63)) for _ in range(roles)]
    else:
        phases = [4 * data.draw(st.integers(0, 255)) for _ in range(roles)]
    check_plan(sizes, W, phases)


def with_env(name, value, fn):
    old = os.environ.get(name)
    os.environ[name] = str(value)
    try:
        return fn()
    finally:
        if old is None:
            os.environ.pop(name)
        else:
            os.environ[name] = old


@pytest.mark.parametrize("phase", [0, 512, 16, 1040, 65536 - 16, 32768, 4])
def test_two_half_tiles_cover_aligned_blocks_only(phase):
    """Tensors longer than a 64 KiB block whose arrays share their offset from a block boundary."""
    sizes = [16384 * 3 + 77, 16384, 16383, 20000, 100, 16384 * 2]
    W = 2
    chunks = check_plan(sizes, W, [phase] * 6)
    assert any(c[4] for c in chunks) == (phase % 16 == 0)


def test_arrays_with_different_block_offsets_get_contiguous_tiles():
    sizes = [16384 * 4]
    chunks = check_plan(sizes, 1, [0, 0, 0, 1024])     # local weights 1 KiB off the others
    assert not any(c[4] for c in chunks) and len(chunks) == 256
    chunks = check_plan(sizes, 1, [1024] * 4)           # all 1 KiB off: blocks start 63 KiB in
    assert sum(1 for c in chunks if c[4]) == 3 * 64


def test_pair_bit_override():
    sizes = [16384 * 4 + 5]
    off = with_env("ODSGD_PAIR_BIT", 0, lambda: check_plan(sizes, 1, [0] * 4, pair_bit=0))
    assert not any(c[4] for c in off)
    bit14 = with_env("ODSGD_PAIR_BIT", 14, lambda: B.odsgd_plan_host(sizes, *fake_layout(sizes, 1, [0] * 4), 1)[1])
    assert {c[4] for c in bit14} == {0, (1 << 14) // 16 - 32}
    covered = sorted(r for c in bit14 for r in B.chunk_elements(c))
    assert covered[0][0] == 0 and covered[-1][1] == sizes[0]
    assert all(a[1] == b[0] for a, b in zip(covered, covered[1:]))


def test_tensor_longer_than_one_row():
    """2^29 + 2^14 + 3 elements: two pointer-table rows, the second advanced by 2 GiB."""
    n = B.ROW_ELEMS + 16384 + 3
    region = lambda j: [0x7f0000000000 + j * (1 << 40)]
    w, v, g, u = region(0), region(1), [region(2)], [region(3)]
    rows, chunks = B.odsgd_plan_host([n], w, v, g, u, 1)
    assert len(rows) == 2 and rows[1][0] == w[0] + 4 * B.ROW_ELEMS and rows[1][3] == u[0][0] + 4 * B.ROW_ELEMS
    assert len(chunks) == -(-n // 256)
    assert max(c[3] for c in chunks) < B.ROW_ELEMS
    total = {0: 0, 1: 0}
    for c in chunks:
        total[c[0]] += c[2]
    assert total == {0: B.ROW_ELEMS, 1: 16384 + 3}
    tail = [c for c in chunks if c[2] < 256]
    assert tail == [(1, True, 3, 16384, 0)]


@pytest.mark.parametrize("name", ["lenet5", "resnet20", "resnet50", "vgg16"])
def test_named_workloads(name):
    w = wl.WORKLOADS[name]
    sizes = wl.numels(w)
    chunks = check_plan(sizes, w.num_workers, [0] * (2 + 2 * w.num_workers))
    assert len(chunks) == sum((n + 255) // 256 for n in sizes)   # tile-aligned bases: no head chunks
    assert sum(c[2] for c in chunks) == wl.total_params(w)
    if name != "lenet5":   # lenet5 has no tensor as long as one 64 KiB block
        assert any(c[4] for c in chunks)


def test_plan_rejects_what_init_rejects():
    w, v, g, u = fake_layout([100], 1, [0, 0, 0, 0])
    with pytest.raises(B.OdsgdError) as e:
        B.odsgd_plan_host([100], w, w, g, u, 1)          # momentum aliases the weights
    assert e.value.code == B.ODSGD_EALIAS
    with pytest.raises(B.OdsgdError) as e:
        B.odsgd_plan_host([100], [w[0] + 2], v, g, u, 1)
    assert e.value.code == B.ODSGD_EALIGN


def test_host_code_under_address_and_undefined_behaviour_sanitizers(tmp_path):
    """Compile the library's host code with ASan + UBSan (device code untouched) together
    with a driver that builds plans for hundreds of random shapes / alignments / error
    cases; it must finish clean."""
    import shutil
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    hipcc = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")
    if not (os.path.exists(hipcc) or shutil.which(hipcc)):
        pytest.skip("hipcc not available")
    exe = str(tmp_path / "plan_sanitized")
    cmd = [hipcc, "--offload-arch=gfx950", "-O1", "-g", "-std=c++17", "-ffp-contract=off",
           "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops",
           "-Xarch_host", "-fsanitize=address", "-Xarch_host", "-fsanitize=undefined",
           "-Xarch_host", "-fno-sanitize-recover=undefined",
           "-I", os.path.join(root, "include"),
           os.path.join(root, "paper_2005_06728_amd", "csrc", "odsgd.hip"),
           "-x", "c++", os.path.join(root, "tests", "plan_sanitizer_driver.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="verify_asan_link_order=0:detect_leaks=1")
    r = subprocess.run([exe], env=env, capture_output=True, text=True, timeout=120)
    assert r.returncode == 0, r.stdout + r.stderr
    assert r.stdout.startswith("ok plans=")
