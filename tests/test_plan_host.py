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


def check_plan(sizes, W, phases, chunk_elems=256):
    w, v, g, u = fake_layout(sizes, W, phases)
    rows, chunks = B.odsgd_plan_host(sizes, w, v, g, u, W)
    K = len(sizes)
    # pointer table
    for k in range(K):
        assert rows[k][:2 + 2 * W] == [w[k], v[k]] + [g[m][k] for m in range(W)] + [u[m][k] for m in range(W)]
        assert rows[k][2 + 2 * W:] == [0] * W
    # coverage: exactly once
    per_tensor = {k: [] for k in range(K)}
    seen_ragged = False
    for t, vec, cnt, off in chunks:
        assert 0 <= t < K and 0 < cnt <= chunk_elems
        per_tensor[t].append((off, cnt, vec))
        if cnt < chunk_elems:
            seen_ragged = True
        else:
            assert not seen_ragged, "a full chunk after a ragged one"
    for k in range(K):
        pieces = sorted(per_tensor[k])
        pos = 0
        for off, cnt, vec in pieces:
            assert off == pos
            pos += cnt
        assert pos == sizes[k]
        all_ptrs = [w[k], v[k]] + [g[m][k] for m in range(W)] + [u[m][k] for m in range(W)]
        vec_ok = all(p % 16 == 0 for p in all_ptrs)
        same_phase = len({p % 1024 for p in all_ptrs}) == 1
        for i, (off, cnt, vec) in enumerate(pieces):
            assert vec == vec_ok
            if vec_ok and same_phase and sizes[k] > 0:
                start = w[k] + 4 * off
                if i > 0 or w[k] % 1024 == 0:
                    assert start % 1024 == 0, "chunk does not start on a tile boundary"
                else:  # head chunk: runs up to the first boundary (or to the end of a short tensor)
                    assert (start + 4 * cnt) % 1024 == 0 or cnt == sizes[k]
    assert len(chunks) <= sum((n + chunk_elems - 1) // chunk_elems + (1 if n else 0) for n in sizes)
    return chunks


@settings(max_examples=150, deadline=None)
@given(sizes=st.lists(st.one_of(st.integers(0, 40), st.integers(200, 1400), st.integers(4000, 9000)),
                      min_size=1, max_size=7),
       W=st.integers(1, 5),
       phase_kind=st.sampled_from(["aligned", "same16", "same4", "mixed16", "mixed4"]),
       data=st.data())
def test_every_element_is_covered_exactly_once(sizes, W, phase_kind, data):
    roles = 2 + 2 * W
    if phase_kind == "aligned":
        phases = [0] * roles
    elif phase_kind == "same16":
        phases = [16 * data.draw(st.integers(1, 63))] * roles
    elif phase_kind == "same4":
        phases = [4 * data.draw(st.integers(1, 255))] * roles
    elif phase_kind == "mixed16":
        phases = [16 * data.draw(st.integers(0, 63)) for _ in range(roles)]
    else:
        phases = [4 * data.draw(st.integers(0, 255)) for _ in range(roles)]
    check_plan(sizes, W, phases)


@pytest.mark.parametrize("chunk", [256, 512, 4096])
def test_chunk_size_override(chunk):
    old = os.environ.get("ODSGD_CHUNK_ELEMS")
    os.environ["ODSGD_CHUNK_ELEMS"] = str(chunk)
    try:
        chunks = check_plan([10000, 3, 0, 4096, 777], 3, [48] * 8, chunk_elems=chunk)
        assert max(c[2] for c in chunks) == chunk
    finally:
        if old is None:
            os.environ.pop("ODSGD_CHUNK_ELEMS")
        else:
            os.environ["ODSGD_CHUNK_ELEMS"] = old


@pytest.mark.parametrize("name", ["lenet5", "resnet20", "resnet50", "vgg16"])
def test_named_workloads(name):
    w = wl.WORKLOADS[name]
    sizes = wl.numels(w)
    chunks = check_plan(sizes, w.num_workers, [0] * (2 + 2 * w.num_workers))
    assert len(chunks) == sum((n + 255) // 256 for n in sizes)   # tile-aligned bases: no head chunks
    assert sum(c[2] for c in chunks) == wl.total_params(w)


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
