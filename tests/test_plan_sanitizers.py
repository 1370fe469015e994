"""The plan builder (host C++) under AddressSanitizer and UndefinedBehaviorSanitizer.

plan.cpp holds no GPU code, so it is compiled here with g++ together with a small driver
(tests/plan_sanitize.cpp) that builds fragments, descriptors and tiles for valid and invalid
shapes.  Any out-of-bounds access, signed overflow or leak aborts the driver."""

import os
import shutil
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


SPEC_FIELDS = ("family", "L", "H", "nq", "nkv", "d", "I", "V", "qkv_bias", "has_embeddings", "E", "Ie", "n_shared",
               "q_lora", "kv_lora", "nope", "rope", "v_dim", "elem_bytes", "tied_embeddings")
LAYOUT_FIELDS = ("kind", "tp", "pp", "ep", "expert_layout", "tp_filter", "ep_filter", "vpp", "first_stage_layers",
                 "last_stage_layers", "vocab_padded", "etp")
CODES = {"dense_gqa": 0, "moe_gqa": 1, "moe_mla": 2, "train": 0, "gen": 1, "per_expert": 0, "grouped": 1}


def case_line(expect, spec, src, dst):
    vals = [expect] + [spec[k] for k in SPEC_FIELDS] + [src[k] for k in LAYOUT_FIELDS] + [dst[k] for k in LAYOUT_FIELDS]
    return " ".join(str(CODES.get(v, v)) for v in vals)


_BUILT = {}


def build(tmp_path):
    if "plan_sanitize" in _BUILT:  # both tests of this module run the same binary
        return _BUILT["plan_sanitize"]
    import tempfile

    exe = os.path.join(tempfile.mkdtemp(prefix="plan_sanitize_"), "plan_sanitize")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan",  # no dependence on the order of preloaded libraries
           "-I" + os.path.join(ROOT, "include"), "-I" + os.path.join(ROOT, "paper_2507_19017_amd", "csrc"),
           os.path.join(ROOT, "paper_2507_19017_amd", "csrc", "plan.cpp"), os.path.join(ROOT, "tests", "plan_sanitize.cpp"),
           "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    _BUILT["plan_sanitize"] = (exe, env)
    return exe, env


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_random_and_mutated_cases_under_asan_and_ubsan(tmp_path):
    """The random workloads (which must be accepted) and mutations of them (one field of the
    shape or of a layout replaced by a random small, zero or negative value: accepted or refused,
    never a crash, an overflow or a tile outside its buffer)."""
    import random

    from synth_inputs import MID, random_case

    # mid-size shapes whose side-by-side merges are also cut as gathered tiles, and wide random ones
    lines = [case_line(1, w["spec"], w["src"], w["dst"]) for w in list(MID.values()) + [random_case(seed, 16) for seed in range(16)]]
    for seed in range(120):
        w = random_case(seed, 1 if seed < 96 else 4)
        lines.append(case_line(1, w["spec"], w["src"], w["dst"]))
        r = random.Random(seed)
        for _ in range(4):
            spec, src, dst = dict(w["spec"]), dict(w["src"]), dict(w["dst"])
            target = r.choice([spec, spec, src, dst])
            key = r.choice([k for k in target if k not in ("family", "kind", "expert_layout")])
            target[key] = r.choice([-1, 0, 1, 2, 3, 5, 7, 8, 12, 16, 33, 64])
            lines.append(case_line(-1, spec, src, dst))
    path = tmp_path / "cases.txt"
    path.write_text("\n".join(lines) + "\n")
    exe, env = build(tmp_path)
    res = subprocess.run([exe, str(path)], capture_output=True, text=True, env=env, timeout=600)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "620 cases from file" in res.stdout and res.stdout.strip().endswith("ok")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_plan_builder_is_clean_under_asan_and_ubsan(tmp_path):
    exe, env = build(tmp_path)
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok")


@pytest.mark.skipif(shutil.which("g++") is None, reason="g++ not available")
def test_c_abi_flows_are_clean_under_asan_and_ubsan(tmp_path):
    """api.cpp (plan lifetime, state machine, swap path, ledger) built against a stand-in HIP runtime
    (tests/fake_hip: device memory is host memory, events are heap objects) with the two launch
    functions replaced by a host interpreter of the tile table: one-shot and streaming flows, every
    refusal, a pinned allocation failing half way, destroy with copies pending.  The sanitizers
    watch every allocation, copy and free; the leak checker sees anything not given back."""
    exe = str(tmp_path / "api_sanitize")
    csrc = os.path.join(ROOT, "paper_2507_19017_amd", "csrc")
    cmd = ["g++", "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-static-libasan", "-static-libubsan", "-I" + os.path.join(ROOT, "tests", "fake_hip"),
           "-I" + os.path.join(ROOT, "include"), "-I" + csrc, os.path.join(csrc, "plan.cpp"), os.path.join(csrc, "api.cpp"),
           os.path.join(ROOT, "tests", "api_sanitize.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=300)
    assert res.returncode == 0, res.stdout + res.stderr
    assert res.stdout.strip().endswith("ok")


@pytest.mark.skipif(not os.path.exists("/opt/rocm/llvm/bin/clang++"), reason="ROCm clang++ not available")
def test_the_real_kernels_run_on_the_host_under_asan(tmp_path):
    """repack.hip itself, compiled for the host against tests/host_simt (a host thread per lane, real
    barriers, __shared__ as statics) and run under AddressSanitizer on small workloads that reach
    the copy kernels (one tile per workgroup and persistent), the register-transpose kernel at
    every element size and the generic transpose: every global and LDS access of the kernels' own
    index arithmetic is checked against the exact extents of the buffers, and every result against
    the descriptor table."""
    exe = str(tmp_path / "kernels_on_host")
    csrc = os.path.join(ROOT, "paper_2507_19017_amd", "csrc")
    cmd = ["/opt/rocm/llvm/bin/clang++", "-std=c++17", "-O0", "-gline-tables-only",  # the many kernel instances compile fast this way
           "-fsanitize=address,undefined", "-fno-sanitize-recover=all",
           "-pthread", "-I" + os.path.join(ROOT, "tests", "host_simt"), "-I" + os.path.join(ROOT, "include"), "-I" + csrc,
           os.path.join(csrc, "plan.cpp"), os.path.join(csrc, "api.cpp"), "-x", "c++", os.path.join(csrc, "repack.hip"),
           os.path.join(ROOT, "tests", "kernels_on_host.cpp"), "-o", exe]
    subprocess.run(cmd, check=True, capture_output=True, text=True)
    env = dict(os.environ)
    env["ASAN_OPTIONS"] = "detect_leaks=1:abort_on_error=0"
    res = subprocess.run([exe], capture_output=True, text=True, env=env, timeout=900)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert res.stdout.strip().endswith("ok") and "element size 8 done" in res.stdout
    # the random small workloads as well: every layout option, odd widths, narrow vector units
    from synth_inputs import random_case

    path = tmp_path / "cases.txt"
    path.write_text("\n".join(case_line(1, w["spec"], w["src"], w["dst"]) for w in (random_case(seed) for seed in range(24))) + "\n")
    res = subprocess.run([exe, str(path)], capture_output=True, text=True, env=env, timeout=900)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "24 cases from file" in res.stdout and res.stdout.strip().endswith("ok")
    # and at the DEFAULT launch shape (1024 lanes, woven order): the tiny models, which include plans with
    # unused buffers (the tile records index a table of the used buffers only), and random ones
    from synth_inputs import TINY

    wls = [w for n, w in sorted(TINY.items()) if n != "big_moe_grouped"] + [random_case(seed) for seed in range(24, 40)]
    path.write_text("\n".join(case_line(1, w["spec"], w["src"], w["dst"]) for w in wls) + "\n")
    res = subprocess.run([exe, str(path), "default"], capture_output=True, text=True, env=env, timeout=900)
    assert res.returncode == 0, res.stdout[-3000:] + res.stderr[-3000:]
    assert "%d cases from file" % len(wls) in res.stdout and res.stdout.strip().endswith("ok")
