"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, sizes its workspace, names its error codes, and rejects bad arguments before
any launch."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "a3po.h")


@pytest.fixture(scope="module")
def lib():
    import paper_2512_06547_amd as a3po
    if not os.path.exists(a3po.lib_path()):
        from paper_2512_06547_amd import build
        build.build(force=True)
    return a3po.lib()


def declared_symbols():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(a3po_[a-z0-9_]+)\s*\(", text)))


def test_header_declares_the_expected_entry_points():
    names = declared_symbols()
    for must in ("a3po_token_logprobs", "a3po_proximal_interp", "a3po_loss_fwd_bwd", "a3po_grpo_advantages",
                 "a3po_workspace_bytes", "a3po_strerror"):
        assert must in names


def test_library_exports_every_declared_symbol(lib):
    for name in declared_symbols():
        assert hasattr(lib, name), name


def test_binding_covers_every_declared_symbol():
    from paper_2512_06547_amd import binding
    assert sorted(binding._SIGNATURES) == declared_symbols()


def test_workspace_size_and_error_strings(lib):
    import paper_2512_06547_amd as a3po
    assert a3po.workspace_bytes(0) >= 256
    small, big = a3po.workspace_bytes(1000, 32000), a3po.workspace_bytes(131072, 151936)
    assert small % 256 == 0 and big % 256 == 0 and big > small
    assert big >= 131072 * (16 + 4 + 4 + 1)
    for code in range(-7, 1):
        assert "unknown" not in a3po.strerror(code)
    assert "unknown" in a3po.strerror(-99)


def test_host_validation_rejects_bad_arguments_before_launch(lib):
    # every call below must return at validation: no device pointer is ever dereferenced
    fake = ctypes.c_void_p(0x1000)
    tl = lib.a3po_token_logprobs
    assert tl(fake, 7, 1, 8, 8, fake, fake, None, None, None) == -3          # dtype
    assert tl(fake, 0, -1, 8, 8, fake, fake, None, None, None) == -2         # T < 0
    assert tl(fake, 0, 1, 0, 8, fake, fake, None, None, None) == -2          # V <= 0
    assert tl(fake, 0, 1, 9, 8, fake, fake, None, None, None) == -2          # ld < V
    assert tl(fake, 0, (1 << 40) + 1, 8, 8, fake, fake, None, None, None) == -2      # more rows than any memory holds
    assert tl(fake, 0, 1, 8, (1 << 40) + 8, fake, fake, None, None, None) == -2      # a stride that would overflow byte offsets
    assert tl(fake, 0, 1, 1 << 31, 1 << 31, fake, fake, None, None, None) == -2       # ids are int32
    assert tl(None, 0, 1, 8, 8, fake, fake, None, None, None) == -1          # null logits
    assert tl(ctypes.c_void_p(0x1002), 0, 1, 8, 8, fake, fake, None, None, None) == -4   # not element aligned
    assert tl(fake, 0, 1, 8, 8, None, fake, None, None, None) == -1          # null chosen
    assert tl(fake, 0, 0, 8, 8, None, None, None, None, None) == 0           # T == 0 is success
    pi = lib.a3po_proximal_interp
    assert pi(None, fake, fake, 1, 4, fake, None, None) == -1
    assert pi(fake, fake, fake, 1, -4, fake, None, None) == -2
    assert pi(None, None, None, 1, 0, None, None, None) == 0
    ga = lib.a3po_grpo_advantages
    assert ga(fake, 7, 4, 1e-6, fake, 10, fake, None) == -2                  # S % G != 0
    assert ga(fake, 8, 0, 1e-6, fake, 10, fake, None) == -2
    assert ga(fake, 8, 4, -1.0, fake, 10, fake, None) == -7
    assert ga(None, 8, 4, 1e-6, fake, 10, fake, None) == -1
    lf = lib.a3po_loss_fwd_bwd
    base = [fake, 1, 4, 64, 64, fake, fake, fake, 3, fake, fake, 0.2, 0.0, fake, fake, None, fake, None,
            ctypes.c_void_p(0x10000), 1 << 20, None]

    def call(**kw):
        a = list(base)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return lf(*a)

    assert call(a11=1.5) == -7 and call(a11=-0.1) == -7 and call(a12=float("nan")) == -7
    assert call(a16=None) == -1 and call(a13=None) == -1 and call(a9=None) == -1
    assert call(a19=16) == -5 and call(a18=None) == -5
    assert call(a18=ctypes.c_void_p(0x10010)) == -4
    assert call(a13=ctypes.c_void_p(0x1001)) == -4 and call(a0=ctypes.c_void_p(0x1001)) == -4
    assert call(a1=2) == -3 and call(a4=32) == -2
    # rows are dealt out through a 32-bit counter: a row count it cannot hold is refused (reachable with a tiny V)
    assert call(a2=(1 << 32) - (1 << 16) + 1, a3=1, a4=8) == -2 and call(a2=1 << 33, a3=1, a4=8) == -2
    assert call(a2=(1 << 32) - (1 << 16), a3=1, a4=8) == -5              # the largest count passes this check


def test_lmhead_entry_points_validate_before_launch(lib):
    fake, ws = ctypes.c_void_p(0x1000), ctypes.c_void_p(0x10000)
    lp = lib.a3po_fused_lmhead_logprob
    # (hidden, weight, T, H, V, chosen, logp, lse, workspace, bytes, stream)
    assert lp(fake, fake, 0, 64, 8, None, None, None, None, 0, None) == 0                 # T == 0 is success
    assert lp(fake, fake, 4, 96, 8, fake, fake, None, ws, 1 << 20, None) == -2            # H not a multiple of 64
    assert lp(fake, fake, 4, (1 << 20) + 64, 8, fake, fake, None, ws, 1 << 20, None) == -2    # H above the limit
    assert lp(fake, fake, 4, 64, 0, fake, fake, None, ws, 1 << 20, None) == -2
    assert lp(fake, fake, 4, 64, 1 << 31, fake, fake, None, ws, 1 << 20, None) == -2      # ids are int32
    assert lp(None, fake, 4, 64, 8, fake, fake, None, ws, 1 << 20, None) == -1
    assert lp(fake, fake, 4, 64, 8, fake, None, None, ws, 1 << 20, None) == -1
    assert lp(ctypes.c_void_p(0x1008), fake, 4, 64, 8, fake, fake, None, ws, 1 << 20, None) == -4
    assert lp(fake, fake, 4, 64, 8, fake, fake, None, ws, 16, None) == -5
    assert lp(fake, fake, 4, 64, 8, fake, fake, None, ctypes.c_void_p(0x10010), 1 << 20, None) == -4
    lf = lib.a3po_fused_lmhead_loss_fwd_bwd
    # (hidden, weight, T, H, V, chosen, logp_behav, versions, cur, adv, mask, eps, denom, dh, dW, logp, prox, loss,
    #  stats, workspace, bytes, stream)
    base = [fake, fake, 4, 64, 8, fake, fake, fake, 3, fake, fake, 0.2, 0.0, fake, fake, fake, None, fake, None,
            ws, 16, None]

    def call(**kw):
        a = list(base)
        for k, v in kw.items():
            a[int(k[1:])] = v
        return lf(*a)

    assert call() == -5                                                                   # workspace too small
    assert call(a3=12) == -2 and call(a4=12) == -2 and call(a3=(1 << 20) + 8) == -2        # H % 8, V % 8, H limit
    assert call(a11=1.0) == -7 and call(a12=float("nan")) == -7
    assert call(a17=None) == -1 and call(a1=None) == -1 and call(a14=None) == -1 and call(a5=None) == -1
    assert call(a13=ctypes.c_void_p(0x1008)) == -4


def test_histogram_validates_before_launch(lib):
    fake = ctypes.c_void_p(0x1000)
    hg = lib.a3po_histogram      # (values, select, T, edges, nbins, accumulate, counts_out, stream)
    assert hg(fake, None, -1, fake, 8, 0, fake, None) == -2
    assert hg(fake, None, 4, fake, 0, 0, fake, None) == -2 and hg(fake, None, 4, fake, 1025, 0, fake, None) == -2
    assert hg(fake, None, 4, fake, 8, 2, fake, None) == -7
    assert hg(None, None, 4, fake, 8, 0, fake, None) == -1 and hg(fake, None, 4, None, 8, 0, fake, None) == -1
    assert hg(fake, None, 4, fake, 8, 0, None, None) == -1


def test_ex_entry_point_validates_its_options_before_launch(lib):
    from paper_2512_06547_amd.binding import LossOptions
    fake = ctypes.c_void_p(0x1000)
    base = [fake, 1, 4, 64, 64, fake, fake, fake, 3, fake, fake, 0.2, 0.0, fake, fake, None, fake, None,
            ctypes.c_void_p(0x10000), 1 << 20, None]
    ex = lib.a3po_loss_fwd_bwd_ex

    def call(opt, versions=fake):
        a = list(base)
        a[7] = versions
        return ex(*a, ctypes.byref(opt))

    assert call(LossOptions(prox_mode=3)) == -7 and call(LossOptions(prox_mode=-1)) == -7
    assert call(LossOptions(prox_mode=0, accumulate=2)) == -7
    assert call(LossOptions(prox_mode=1)) == -1                          # given-prox without the array
    assert call(LossOptions(prox_mode=0), versions=None) == -1           # interpolation needs versions
    te = lib.a3po_token_logprobs_entropy
    assert te(fake, 0, 1, 8, 8, fake, fake, None, None, None, None) == -1   # entropy_out is required
    assert te(fake, 0, 0, 8, 8, None, None, None, None, None, None) == 0
    assert te(fake, 5, 1, 8, 8, fake, fake, None, None, fake, None) == -3


def _check_plan_invariants(seq_len, n_mb, budget, first, owner):
    """What any correct plan must satisfy, checked by brute force (independent of how it was produced)."""
    S = len(seq_len)
    assert first[0] == (0 if len(owner) else S) and first[-1] == S and len(first) == len(owner) + 1
    assert all(a <= b for a, b in zip(first, first[1:])) and all(a <= b for a, b in zip(owner, owner[1:]))
    for i, k in enumerate(owner):
        lo, hi = k * S // n_mb, (k + 1) * S // n_mb
        a, b = first[i], first[i + 1]
        assert lo <= a < b <= hi, "a micro-batch holds at least one sequence and stays inside its mini-batch"
        tok = sum(seq_len[a:b])
        nonempty = [s for s in range(a, b) if seq_len[s] > 0]
        assert tok <= budget or len(nonempty) == 1, "budget respected unless a single sequence exceeds it"
        if i + 1 < len(owner) and owner[i + 1] == k:   # greedy: the sequence that opened the next one did not fit
            nxt = first[i + 1]
            assert seq_len[nxt] > 0 and tok + seq_len[nxt] > budget
    covered = sorted(s for i in range(len(owner)) for s in range(first[i], first[i + 1]))
    assert covered == [s for k in range(n_mb) for s in range(k * S // n_mb, (k + 1) * S // n_mb)] == list(range(S))


def test_microbatch_planner_against_reference_and_invariants(lib):
    import numpy as np
    import oracle
    import paper_2512_06547_amd as a3po
    # hand-worked: budget 10, two mini-batches of three sequences each
    first, owner = a3po.plan_microbatches([4, 5, 3, 12, 0, 2], 2, 10)
    assert first.tolist() == [0, 2, 3, 5, 6] and owner.tolist() == [0, 0, 1, 1]   # the empty sequence rides with the oversize one
    rng = np.random.default_rng(3)
    for trial in range(300):
        S = int(rng.integers(0, 40))
        n_mb = int(rng.integers(1, 7))
        budget = int(rng.integers(1, 60))
        lens = rng.integers(0, 40, size=S)
        lens[rng.random(S) < 0.15] = 0
        first, owner = a3po.plan_microbatches(lens, n_mb, budget)
        rf, ro = oracle.plan_microbatches(lens, n_mb, budget)
        assert first.tolist() == rf and owner.tolist() == ro, (lens, n_mb, budget)
        _check_plan_invariants(lens.tolist(), n_mb, budget, rf, ro)
    # the paper's first setup: 1,024 sequences of at most 1,024 tokens, 4 updates, 10,240 tokens per pass
    lens = rng.integers(64, 1025, size=1024)
    first, owner = a3po.plan_microbatches(lens, 4, 10240)
    _check_plan_invariants(lens.tolist(), 4, 10240, first.tolist(), owner.tolist())
    assert np.bincount(owner, minlength=4).min() > 0
    # errors: nothing fits in a capacity that is too small, bad sizes
    with pytest.raises(a3po.A3poError) as e:
        a3po.plan_microbatches([5, 5, 5, 5], 1, 5, capacity=3)
    assert e.value.code == -2
    for bad in (dict(n_minibatches=0, max_tokens=5), dict(n_minibatches=2, max_tokens=0)):
        with pytest.raises(a3po.A3poError):
            a3po.plan_microbatches([1, 2], **bad)
    with pytest.raises(a3po.A3poError):
        a3po.plan_microbatches([1, -2], 1, 5)


C_PROGRAM = r"""
#include <stddef.h>
#include <stdio.h>
#include <string.h>
#include "a3po.h"

int main(void)
{
    /* host-only entry points: nothing here touches a GPU */
    const int64_t seq_len[5] = {7, 3, 9, 0, 4};
    int64_t first[8];
    int32_t owner[7];
    int64_t n = -1;
    a3po_loss_options opt;
    a3po_stats st;
    memset(&opt, 0, sizeof opt);
    memset(&st, 0, sizeof st);
    if (a3po_plan_microbatches(seq_len, 5, 2, 10, first, owner, 7, &n) != A3PO_OK) return 1;
    printf("micro %lld:", (long long)n);
    for (int64_t i = 0; i <= n; ++i) printf(" %lld", (long long)first[i]);
    printf("\n");
    printf("ws %zu\n", a3po_workspace_bytes(A3PO_WS_LOSS_FWD_BWD, 1000, 32000, 0));
    printf("err %s\n", a3po_strerror(A3PO_E_WORKSPACE));
    /* a null logits pointer is refused on the host, before any launch */
    printf("null %d\n", a3po_token_logprobs(NULL, A3PO_BF16, 4, 64, 64, NULL, NULL, NULL, NULL, NULL));
    printf("sizes %zu %zu %zu\n", sizeof(a3po_stats), sizeof(a3po_shard_partial), sizeof(a3po_loss_options));
    printf("offsets %zu %zu %zu %zu\n", offsetof(a3po_stats, iw_min), offsetof(a3po_stats, entropy_mean),
           offsetof(a3po_loss_options, logp_prox_in), offsetof(a3po_loss_options, denom_dev));
    return (int)(opt.accumulate + st.n_tokens);
}
"""


def test_header_is_plain_c_and_the_library_links_from_c(lib, tmp_path):
    """include/a3po.h compiles as strict C99 and a C program linked against the library gets the same answers
    as the Python binding (planner, workspace size, error strings, host-side validation)."""
    import shutil
    import subprocess

    import numpy as np
    import paper_2512_06547_amd as a3po
    cc = shutil.which("gcc") or shutil.which("cc")
    if cc is None:
        pytest.skip("no C compiler")
    src = tmp_path / "use_a3po.c"
    src.write_text(C_PROGRAM)
    exe = tmp_path / "use_a3po"
    libdir = os.path.dirname(a3po.lib_path())
    subprocess.run([cc, "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(ROOT, "include"),
                    str(src), "-o", str(exe), "-L", libdir, "-la3po", f"-Wl,-rpath,{libdir}", "-Wl,-rpath,/opt/rocm/lib"],
                   check=True, capture_output=True, text=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True, timeout=120).stdout.splitlines()
    first, owner = a3po.plan_microbatches(np.array([7, 3, 9, 0, 4], dtype=np.int64), 2, 10)
    assert out[0] == f"micro {len(owner)}: " + " ".join(str(int(x)) for x in first)
    assert out[1] == f"ws {a3po.workspace_bytes(1000, 32000)}"
    assert out[2] == "err " + lib.a3po_strerror(-5).decode()
    assert out[3] == "null -1"
    # struct layouts as the binding mirrors them
    B = a3po.binding
    assert out[4] == f"sizes {B.STATS_DTYPE.itemsize} 16 {ctypes.sizeof(B.LossOptions)}"
    assert out[5] == (f"offsets {B.STATS_DTYPE.fields['iw_min'][1]} {B.STATS_DTYPE.fields['entropy_mean'][1]} "
                      f"{B.LossOptions.logp_prox_in.offset} {B.LossOptions.denom_dev.offset}")


def test_library_needs_only_the_hip_runtime(lib):
    """No vendor math library is linked: the dynamic section names the HIP runtime and the C / C++ run-times only."""
    import shutil
    import subprocess
    if shutil.which("readelf") is None:
        pytest.skip("needs readelf")
    from paper_2512_06547_amd import binding
    out = subprocess.run(["readelf", "-d", binding.lib_path()], check=True, capture_output=True, text=True).stdout
    needed = [ln.split("[")[1].split("]")[0] for ln in out.splitlines() if "(NEEDED)" in ln]
    assert any(n.startswith("libamdhip64") for n in needed)
    allowed = ("libamdhip64", "libstdc++", "libm.", "libgcc_s", "libc.", "ld-linux", "libpthread", "libdl", "librt")
    assert all(n.startswith(allowed) for n in needed), needed


def test_host_code_is_clean_under_address_and_undefined_behaviour_sanitizers(lib, tmp_path):
    """The translation unit that holds the library's host logic (planner, workspace sizes, validation of every
    entry point) is rebuilt with -fsanitize=address,undefined on the host side and linked with the other objects
    as built; a driver compiled the same way runs 100,000 random plans into exactly-sized arrays and every
    refusal path.  Device code is untouched (sanitizers are host-only here)."""
    import glob
    import subprocess
    from paper_2512_06547_amd import build
    clang = os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(build.HIPCC))), "llvm", "bin", "clang")
    others = [o for o in glob.glob(os.path.join(build.OBJ, "*.hip.o")) if not o.endswith("a3po_api.hip.o")]
    if not os.path.exists(clang) or len(others) != len(build.SOURCES) - 1:
        pytest.skip("needs ROCm's clang and the objects of an in-tree build")
    san = ["-fsanitize=address", "-fsanitize=undefined", "-fno-omit-frame-pointer"]
    host_san = [x for f in san for x in ("-Xarch_host", f)]
    flags = [f for f in build.FLAGS if f != "-O3"] + ["-O1", "-g"]
    api_o = str(tmp_path / "a3po_api.san.o")
    subprocess.run([build.HIPCC, *flags, *host_san, "-c", os.path.join(build.CSRC, "a3po_api.hip"), "-o", api_o],
                   check=True, capture_output=True)
    rocm_lib = os.path.join(os.path.dirname(os.path.dirname(os.path.realpath(build.HIPCC))), "lib")
    so = str(tmp_path / "liba3po.so")
    subprocess.run([build.HIPCC, "--offload-arch=gfx950", "-shared", "-fPIC", *san[:2], "-o", so, api_o, *others,
                    f"-Wl,-rpath,{rocm_lib}"], check=True, capture_output=True)
    exe = str(tmp_path / "host_sanitize")
    subprocess.run([clang, "-std=c99", "-g", *san, "-I", os.path.join(ROOT, "include"),
                    os.path.join(ROOT, "tests", "a3po_host_sanitize_driver.c"), "-o", exe, "-L", str(tmp_path), "-la3po",
                    f"-Wl,-rpath,{tmp_path}", f"-Wl,-rpath,{rocm_lib}"], check=True, capture_output=True)
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=0")      # the GPU runtime's own start-up allocations are not ours
    res = subprocess.run([exe], capture_output=True, text=True, timeout=300, env=env)
    assert res.returncode == 0, (res.stdout[-500:], res.stderr[-2000:])
    assert res.stdout.strip().endswith("ok") and "runtime error" not in res.stderr and "ERROR" not in res.stderr
