"""CPU-only checks of the C-ABI library: it loads, exports every symbol the
header declares, and rejects bad arguments on the host before any launch."""
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    import paper_2503_18427_amd as aes
    return aes.library()


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "aes_spmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(aes_[a-z0-9_]+)\s*\(", text)))


def test_header_symbols_exported(lib):
    from paper_2503_18427_amd import binding
    names = _declared_functions()
    assert set(names) == set(binding.SIGNATURES), "binding and header disagree"
    for n in names:
        assert hasattr(lib, n), n


def test_binding_constants_equal_the_headers():
    """Every enumerator of include/aes_spmm.h has the same value under the same name in the binding."""
    import paper_2503_18427_amd as aes
    text = open(os.path.join(ROOT, "include", "aes_spmm.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    found = dict(re.findall(r"\b(AES_[A-Z0-9_]+)\s*=\s*([-0-9 <]+?)\s*[,}\n]", text))
    assert len(found) == 17, found
    for name, expr in found.items():
        assert getattr(aes.binding, name) == eval(expr, {"__builtins__": {}}), name


def test_no_oracle_in_product():
    """The product package must not reach the oracle (or any CPU fallback)."""
    pkg = os.path.join(ROOT, "paper_2503_18427_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".cpp", ".hpp", ".h")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.lower(), f


def test_capacity_and_workspace(lib):
    import paper_2503_18427_amd as aes
    assert aes.aes_sample_capacity(10, 100, 4) == 40
    assert aes.aes_sample_capacity(10, 30, 4) == 30
    assert aes.aes_sample_capacity(10, 100, 0) == 100
    assert aes.aes_sample_capacity(0, 0, 16) == 0
    with pytest.raises(aes.AesError) as e:
        aes.aes_sample_capacity(-1, 5, 4)
    assert e.value.code == -1
    with pytest.raises(aes.AesError):
        aes.aes_sample_capacity(1, 5, (1 << 20) + 1)
    assert aes.aes_sample_workspace_bytes(0) == 8
    assert aes.aes_sample_workspace_bytes(1025) == 8 * 3 + 4 * 32 * 2
    assert aes.aes_quantize_workspace_bytes(1000, 128, aes.AES_Q_PER_ROW) == 0
    assert aes.aes_quantize_workspace_bytes(1000, 128, aes.AES_Q_PER_COLUMN) > 0


def test_argument_errors_are_host_side(lib):
    """Every call below must fail before touching the GPU (there is none here)."""
    import paper_2503_18427_amd as aes
    fake = 0x1000  # never dereferenced: argument checks come first
    sb = lib.aes_sample_build
    assert sb(-1, 1, 0, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert "negative" in aes.aes_last_error()
    assert sb(4, 1 << 31, 0, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, fake, 1 << 20, None) == -2
    assert sb(4, 4, 8, fake, fake, fake, -3, 0, 0, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert sb(4, 4, 8, None, fake, fake, 4, 0, 0, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert sb(4, 4, 8, fake, None, fake, 4, 0, 0, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert sb(4, 4, 8, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, None, 0, None) == -3
    assert sb(4, 4, 8, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, fake, 8, None) == -3
    assert "workspace" in aes.aes_last_error()
    assert sb(4, 4, 8, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, fake + 4, 1 << 20, None) == -3

    assert sb(4, 4, 8, fake, fake, fake, 4, 0, 3, fake, fake, fake, None, None, fake, 1 << 20, None) == -1
    assert "strategy" in aes.aes_last_error()
    na = lib.aes_sample_build_noalloc
    assert na(-1, 1, 0, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, None) == -1
    assert na(4, 4, 8, fake, fake, fake, 4, 0, 3, fake, fake, fake, None, None, None) == -1
    assert na(4, 4, 8, None, fake, fake, 4, 0, 0, fake, fake, fake, None, None, None) == -1
    assert na(aes.AES_NOALLOC_MAX_ROWS + 1, 4, 8, fake, fake, fake, 4, 0, 0, fake, fake, fake, None, None, None) == -2
    assert "built-in scratch" in aes.aes_last_error()
    ff = lib.aes_spmm_fused_f32
    assert ff(4, 4, fake, fake, fake, -1, 0, 0, fake, 8, 8, fake, 8, None) == -1
    assert ff(4, 4, fake, fake, fake, 16, 0, 5, fake, 8, 8, fake, 8, None) == -1
    assert ff(4, 4, None, fake, fake, 16, 0, 0, fake, 8, 8, fake, 8, None) == -1
    assert ff(4, 4, fake, fake, fake, 16, 0, 0, fake, 4, 8, fake, 8, None) == -1
    fq = lib.aes_spmm_fused_q8
    assert fq(4, 4, fake, fake, fake, 16, 0, 0, fake, 8, 8, 9, 1, fake, fake, fake, 8, None) == -1
    assert fq(4, 4, fake, fake, fake, 16, 0, 0, fake, 8, 8, 1, 1, None, fake, fake, 8, None) == -1
    assert fq(4, 4, fake, fake, fake, 1 << 21, 0, 0, fake, 8, 8, 1, 1, fake, fake, fake, 8, None) == -1

    f32 = lib.aes_spmm_f32
    assert f32(-1, 4, 0, fake, fake, fake, None, fake, 8, 8, fake, 8, None) == -1
    assert f32(4, 4, 0, fake, fake, fake, None, fake, 8, 0, fake, 8, None) == -1
    assert f32(4, 4, 0, fake, fake, fake, None, fake, 4, 8, fake, 8, None) == -1      # ldx < F
    assert f32(4, 4, 0, fake, fake, fake, None, fake, 8, 8, fake, 4, None) == -1      # ldy < F
    assert f32(4, 4, 0, None, fake, fake, None, fake, 8, 8, fake, 8, None) == -1
    assert f32(4, 4, 0, fake, fake, fake, None, None, 8, 8, fake, 8, None) == -1
    assert f32(4, 4, 0, fake, fake, fake, None, fake, 8, 8, None, 8, None) == -1
    assert f32(0, 4, 0, fake, fake, fake, None, fake, 8, 8, None, 8, None) == 0       # nothing to do
    assert f32(4, 4, -1, fake, fake, fake, None, fake, 8, 8, fake, 8, None) == -1     # bad W
    assert f32(4, 4, 0, fake, fake, fake, None, fake, 1 << 32, 8, fake, 8, None) == -2  # ldx beyond 32 bits
    assert "32 bits" in aes.aes_last_error()

    q = lib.aes_quantize_features
    assert q(-1, 8, fake, 8, 1, 1, fake, 8, fake, fake, fake, 1 << 20, None) == -1
    assert q(4, 8, fake, 8, 7, 1, fake, 8, fake, fake, fake, 1 << 20, None) == -1
    assert q(4, 8, fake, 8, 1, 9, fake, 8, fake, fake, fake, 1 << 20, None) == -1
    assert q(4, 8, fake, 4, 1, 1, fake, 8, fake, fake, fake, 1 << 20, None) == -1
    assert q(4, 8, fake, 8, 0, 1, fake, 8, fake, None, fake, 1 << 20, None) == -1  # affine needs zero
    assert q(4, 8, fake, 8, 1, 1, fake, 8, fake, None, None, 0, None) == -3
    assert q(4, 8, None, 8, 1, 2, fake, 8, fake, None, None, 0, None) == -1

    dq = lib.aes_dequantize_features
    assert dq(-1, 8, fake, 8, 1, 1, fake, None, fake, 8, None) == -1
    assert dq(4, 8, fake, 4, 1, 1, fake, None, fake, 8, None) == -1
    assert dq(4, 8, fake, 8, 0, 1, fake, None, fake, 8, None) == -1     # affine needs zero
    assert dq(4, 8, fake, 8, 1, 1, None, None, fake, 8, None) == -1
    assert dq(4, 8, None, 8, 1, 1, fake, None, fake, 8, None) == -1
    assert dq(0, 8, None, 8, 1, 1, fake, None, None, 8, None) == 0

    fold = lib.aes_plan_fold_row_constants
    assert fold(-1, fake, fake, fake, 1, fake, None, fake, None, None) == -1
    assert fold(4, fake, fake, fake, 7, fake, None, fake, None, None) == -1
    assert fold(4, None, fake, fake, 1, fake, None, fake, None, None) == -1
    assert fold(4, fake, fake, fake, 1, None, None, fake, None, None) == -1
    assert fold(4, fake, fake, fake, 0, fake, None, fake, fake, None) == -1      # affine needs zero
    assert fold(4, fake, fake, fake, 0, fake, fake, fake, None, None) == -1      # affine needs row_bias
    assert fold(0, fake, fake, fake, 1, fake, None, fake, None, None) == 0
    assert lib.aes_spmm_fused_q8(4, 4, fake, fake, fake, 16, 0, 0, fake, 8, 8, 1, 3, fake, None, fake, 8, None) == -1
    assert lib.aes_quantize_features(4, 8, fake, 8, 1, 3, fake, 8, fake, fake, fake, 1 << 20, None) == -1

    gl = lib.aes_gcn_layer_f32
    assert gl(-1, 4, 0, fake, fake, fake, fake, 8, 8, fake, 8, 8, fake, 8, None) == -1
    assert gl(4, 4, 0, fake, fake, fake, fake, 8, 8, fake, 4, 8, fake, 8, None) == -1      # ldt < Fo
    assert gl(4, 4, 0, fake, fake, fake, fake, 8, 8, None, 8, 8, fake, 8, None) == -1      # Theta NULL
    assert gl(4, 4, 0, fake, fake, fake, fake, 8, 8, fake, 8, 8, None, 8, None) == -1      # H NULL
    assert gl(4, 4, 0, fake, fake, fake, fake, 1 << 24, 1 << 24, fake, 8, 8, fake, 8, None) == -1  # F out of range
    assert gl(4, 4, 0, fake, fake, fake, fake, 1 << 32, 8, fake, 8, 8, fake, 8, None) == -2  # ldx beyond 32 bits
    assert gl(4, 4, 0, fake, fake, fake, fake, 8, 8, fake, 1 << 28, 8, fake, 8, None) == -2  # ldt beyond the lane offsets
    assert gl(0, 4, 0, fake, fake, fake, fake, 8, 8, fake, 8, 8, None, 8, None) == 0

    glq = lib.aes_gcn_layer_q8
    assert glq(4, 4, 0, fake, fake, fake, fake, 8, 8, 9, 1, fake, None, fake, 8, 8, fake, 8, None) == -1   # scheme
    assert glq(4, 4, 0, fake, fake, fake, fake, 8, 8, 1, 7, fake, None, fake, 8, 8, fake, 8, None) == -1   # granularity
    assert glq(4, 4, 0, fake, fake, fake, fake, 8, 8, 1, 1, None, None, fake, 8, 8, fake, 8, None) == -1   # scale NULL
    assert glq(4, 4, 0, fake, fake, fake, fake, 8, 8, 0, 1, fake, None, fake, 8, 8, fake, 8, None) == -1   # affine, zero NULL
    assert glq(0, 4, 0, fake, fake, fake, fake, 8, 8, 1, 1, fake, None, fake, 8, 8, None, 8, None) == 0

    q8 = lib.aes_spmm_q8
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 8, 8, 5, 1, fake, fake, fake, 8, None) == -1
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 8, 8, 1, 5, fake, fake, fake, 8, None) == -1
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 8, 8, 1, 1, None, fake, fake, 8, None) == -1
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 8, 8, 0, 1, fake, None, fake, 8, None) == -1
    assert q8(0, 4, 0, fake, fake, fake, None, fake, 8, 8, 1, 1, fake, None, None, 8, None) == 0

    # per-node constants inside the rows of codes (granularity 4): the layout is checked on the host
    ild = lib.aes_quantize_inline_ld
    assert ild(100, 1) == 128 and ild(124, 1) == 128 and ild(128, 1) == 256 and ild(602, 1) == 640
    assert ild(121, 1) == 128 and ild(121, 0) == 256 and ild(120, 0) == 128
    assert ild(0, 1) == -1 and ild(8, 5) == -1
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 8, 8, 1, 4, None, None, fake, 8, None) == -1       # ldq = 8 < 8 + 4
    assert "inside the rows" in aes.aes_last_error()
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 14, 8, 1, 4, None, None, fake, 8, None) == -1      # ldq % 4
    assert q8(4, 4, 0, fake, fake, fake, None, fake + 2, 16, 8, 1, 4, None, None, fake, 8, None) == -1  # Xq misaligned
    assert q8(4, 4, 0, fake, fake, fake, None, fake, 12, 8, 0, 4, None, None, fake, 8, None) == -1      # affine: 8 more bytes
    assert q(4, 8, fake, 8, 1, 4, fake, 8, None, None, None, 0, None) == -1
    assert dq(4, 8, fake, 8, 1, 4, None, None, fake, 8, None) == -1
    assert glq(4, 4, 0, fake, fake, fake, fake, 8, 8, 1, 4, None, None, fake, 8, 8, fake, 8, None) == -1
    assert lib.aes_spmm_fused_q8(4, 4, fake, fake, fake, 16, 0, 0, fake, 8, 8, 1, 4, None, None, fake, 8, None) == -1


def test_header_and_library_from_plain_c(lib, tmp_path):
    """include/aes_spmm.h is valid C99 and the library links and answers from a C program."""
    import shutil
    import subprocess
    import paper_2503_18427_amd as aes
    if shutil.which("gcc") is None:
        pytest.skip("gcc not available")
    from paper_2503_18427_amd import build as aes_build
    so = aes_build.LIB
    exe = str(tmp_path / "abi_c_client")
    cmd = ["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.join(ROOT, "include"),
           os.path.join(ROOT, "tests", "abi_c_client.c"), "-o", exe, so, "-Wl,-rpath," + os.path.dirname(so)]
    build = subprocess.run(cmd, capture_output=True, text=True)
    assert build.returncode == 0, build.stderr
    run = subprocess.run([exe], capture_output=True, text=True, timeout=120)
    assert run.returncode == 0 and "abi c client ok" in run.stdout, run.stdout + run.stderr


def test_binding_rejects_host_tensors():
    import torch
    import paper_2503_18427_amd as aes
    with pytest.raises(TypeError):
        aes.aes_sample_build(torch.zeros(3, dtype=torch.int64), torch.zeros(2, dtype=torch.int32),
                             torch.zeros(2), 2, 4)


def test_last_error_is_per_thread(lib):
    """The message buffer is thread-local: a failure in one thread does not
    overwrite what another thread reads."""
    import threading
    import paper_2503_18427_amd as aes
    fake = 0x1000
    assert lib.aes_spmm_f32(-1, 4, 0, fake, fake, fake, None, fake, 8, 8, fake, 8, None) == -1
    mine = aes.aes_last_error()
    seen = {}

    def other():
        seen["before"] = aes.aes_last_error()
        lib.aes_quantize_features(-5, 8, fake, 8, 1, 1, fake, 8, fake, fake, fake, 1 << 20, None)
        seen["after"] = aes.aes_last_error()

    t = threading.Thread(target=other)
    t.start()
    t.join()
    assert seen["before"] == "" and "aes_quantize_features" in seen["after"]
    assert aes.aes_last_error() == mine and "aes_spmm_f32" in mine


def test_builtin_scratch_symbol_is_visible_to_the_runtime(lib, tmp_path):
    """The device-side array behind aes_sample_build_noalloc is looked up by name at run time
    (hipGetSymbolAddress); a symbol local to the code object cannot be found and the runtime aborts.
    Checks the device code objects inside the built library: exactly one global `scratch` object."""
    import shutil
    import subprocess
    import paper_2503_18427_amd as aes
    bundler, readelf = "/opt/rocm/llvm/bin/clang-offload-bundler", "/opt/rocm/llvm/bin/llvm-readelf"
    if shutil.which("objcopy") is None or not (os.path.exists(bundler) and os.path.exists(readelf)):
        pytest.skip("binutils / LLVM tools not available")
    fat = tmp_path / "lib.fat"
    subprocess.run(["objcopy", "-O", "binary", "--only-section=.hip_fatbin", aes.build.lib_path(), str(fat)], check=True)
    data = fat.read_bytes()
    magic = b"__CLANG_OFFLOAD_BUNDLE__"
    starts = [m.start() for m in re.finditer(re.escape(magic), data)]
    assert starts, "no device code in the library"
    found = []
    for n, (a, b) in enumerate(zip(starts, starts[1:] + [len(data)])):
        part, co = tmp_path / f"b{n}.fat", tmp_path / f"b{n}.co"
        part.write_bytes(data[a:b])
        subprocess.run([bundler, "--unbundle", "--type=o", f"--input={part}",
                        "--targets=hipv4-amdgcn-amd-amdhsa--gfx950", f"--output={co}"], check=True)
        table = subprocess.run([readelf, "-s", "--dyn-syms", str(co)], capture_output=True, text=True, check=True).stdout
        for line in table.splitlines():
            f = line.split()
            if len(f) >= 8 and f[3] == "OBJECT" and f[7].endswith("scratch"):
                found.append((f[4], int(f[2])))
    assert found, "device array `scratch` is missing from the code objects"
    assert all(bind == "GLOBAL" for bind, _ in found), found
    assert {size for _, size in found} == {8 * (16384 + 1) + 4 * 32 * 16384}, found
