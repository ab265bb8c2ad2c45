"""Host-side checks of the C-ABI library that need no GPU: it loads, exports
every symbol the header declares, sizes messages as Table 3 implies (b bits per
element), and turns every host-checkable mistake into an error code before any
launch."""
import ctypes
import re
from pathlib import Path

import pytest

from paper_2206_01299_amd import binding as B

ROOT = Path(__file__).resolve().parent.parent


def test_library_exports_every_declared_symbol():
    header = (ROOT / "include" / "aqsgd.h").read_text()
    body = re.sub(r"/\*.*?\*/", "", header, flags=re.S)
    declared = set(re.findall(r"\b(aqsgd_[a-z_0-9]+)\s*\(", body))
    assert declared, "no declarations found in the header"
    assert declared == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None
    assert re.fullmatch(r"\d+\.\d+\.\d+", B.version())


def test_desc_layout_matches_header():
    assert ctypes.sizeof(B.Desc) == 48
    assert B.Desc.bits.offset == 24 and B.Desc.rng_seed.offset == 40


def test_message_sizes():
    d = B.make_desc(batch=4, n_per=1024 * 1600, n_samples=8192, bits=4, group=1600, dtype="f16")
    assert B.codes_bytes(d) == 4 * 1024 * 1600 // 2
    assert B.scales_count(d) == 4096
    d = B.make_desc(batch=32, n_per=256 * 1536, n_samples=100_000, bits=3, group=64, dtype="bf16")
    assert B.codes_bytes(d) == 32 * 256 * 1536 * 3 // 8
    assert B.scales_count(d) == 32 * 256 * 1536 // 64
    d = B.make_desc(batch=0, n_per=64, n_samples=1, bits=2, group=64, dtype="f32")
    assert B.codes_bytes(d) == 0 and B.scales_count(d) == 0


BAD = [
    (dict(bits=5), -2), (dict(bits=0), -2), (dict(bits=16), -2), (dict(bits=7), -2),
    (dict(group=0), -3), (dict(group=-8), -3), (dict(group=48), -3),     # 48 does not divide 1600
    (dict(bits=3, group=4, n_per=1600), -3),                              # 12 bits: not whole bytes
    (dict(bits=2, group=2, n_per=1600), -3),
    (dict(dtype_code=7), -4), (dict(rounding=2), -4),
    (dict(batch=-1), -5), (dict(n_per=0), -5), (dict(n_samples=0), -5),
    (dict(n_samples=2**62), -5), (dict(batch=2**31), -5),
]


@pytest.mark.parametrize("change,status", BAD)
def test_bad_descriptors_are_rejected_before_any_launch(change, status):
    kw = dict(batch=4, n_per=1600, n_samples=16, bits=4, group=1600, dtype="f16")
    dtype_code = change.pop("dtype_code", None) if "dtype_code" in change else None
    kw.update({k: v for k, v in change.items()})
    d = B.make_desc(**kw)
    if dtype_code is not None:
        d.dtype = dtype_code
    p = ctypes.c_void_p(4096)          # never dereferenced: the descriptor is refused first
    L = B.lib()
    assert L.aqsgd_encode(ctypes.byref(d), p, p, p, p, p, None) == status
    assert L.aqsgd_decode(ctypes.byref(d), p, p, p, p, p, None) == status
    if "n_samples" not in change:
        assert L.aqsgd_grad_quant(ctypes.byref(d), p, p, p, None) == status
        assert L.aqsgd_grad_dequant(ctypes.byref(d), p, p, p, None) == status
    assert B.strerror(status) != "unknown status"


def test_null_and_misaligned_pointers():
    d = B.make_desc(batch=4, n_per=1600, n_samples=16, bits=4, group=1600, dtype="f16")
    L = B.lib()
    ok = ctypes.c_void_p(4096)
    odd = ctypes.c_void_p(4096 + 2)
    assert L.aqsgd_encode(ctypes.byref(d), None, ok, ok, ok, ok, None) == -1
    assert L.aqsgd_encode(ctypes.byref(d), ok, ok, None, ok, ok, None) == -1
    assert L.aqsgd_decode(ctypes.byref(d), ok, ok, ok, ok, None, None) == -1
    assert L.aqsgd_encode(ctypes.byref(d), odd, ok, ok, ok, ok, None) == -6
    assert L.aqsgd_encode(ctypes.byref(d), ok, ok, odd, ok, ok, None) == -6
    assert L.aqsgd_decode(ctypes.byref(d), ok, ok, ok, ok, odd, None) == -6
    assert L.aqsgd_grad_quant(ctypes.byref(d), ok, odd, ok, None) == -6
    assert L.aqsgd_grad_dequant(ctypes.byref(d), ok, ok, None, None) == -1
    assert L.aqsgd_encode(None, ok, ok, ok, ok, ok, None) == -1
    # an empty call succeeds without looking at the pointers
    d0 = B.make_desc(batch=0, n_per=1600, n_samples=16, bits=4, group=1600, dtype="f16")
    assert L.aqsgd_encode(ctypes.byref(d0), None, None, None, None, None, None) == 0
    assert L.aqsgd_decode(ctypes.byref(d0), None, None, None, None, None, None) == 0


def test_binding_has_no_cpu_route():
    """The binding refuses host tensors instead of computing anything itself."""
    import torch
    d = B.make_desc(batch=1, n_per=64, n_samples=1, bits=4, group=64, dtype="f32")
    t = torch.zeros(64)
    with pytest.raises(ValueError):
        B.encode(d, t, torch.zeros(1, dtype=torch.int64), t, torch.zeros(32, dtype=torch.uint8),
                 torch.zeros(1))
    src = (ROOT / "paper_2206_01299_amd" / "binding.py").read_text()
    assert "import oracle" not in src and "from oracle" not in src


def test_binding_checks_tensor_types_and_sizes_against_the_descriptor(monkeypatch):
    """The kernels index every buffer from the descriptor alone, so a tensor of another
    element type or a smaller size must be refused before its pointer reaches the library
    (an int32 id tensor would be read as int64: garbage rows, out-of-range writes)."""
    import torch
    monkeypatch.setattr(B, "_dev", lambda t, what: ctypes.c_void_p(0))    # host tensors stand in for device ones
    d = B.make_desc(batch=2, n_per=64, n_samples=4, bits=4, group=64, dtype="f16")
    act = torch.zeros((2, 64), dtype=torch.float16)
    ids = torch.zeros(2, dtype=torch.int64)
    m = torch.zeros((4, 64), dtype=torch.float16)
    codes = torch.zeros(B.codes_bytes(d), dtype=torch.uint8)
    scales = torch.zeros(B.scales_count(d), dtype=torch.float32)

    def refused(what, **kw):
        a = dict(act=act, sample_ids=ids, m_buf=m, codes=codes, scales=scales)
        a.update(kw)
        with pytest.raises(ValueError, match=what):
            B.encode(d, a["act"], a["sample_ids"], a["m_buf"], a["codes"], a["scales"])

    refused("sample_ids", sample_ids=ids.to(torch.int32))
    refused("sample_ids", sample_ids=torch.zeros(3, dtype=torch.int64))
    refused("act", act=act.float())
    refused("act", act=torch.zeros((1, 64), dtype=torch.float16))
    refused("m_buf", m_buf=torch.zeros((3, 64), dtype=torch.float16))
    refused("m_buf", m_buf=m.to(torch.bfloat16))
    refused("codes", codes=codes[:-1])
    refused("codes", codes=codes.to(torch.int8))
    refused("scales", scales=scales.double())
    refused("scales", scales=scales[:-1])
    with pytest.raises(ValueError, match="out"):
        B.decode(d, codes, scales, ids, m, torch.zeros((2, 63), dtype=torch.float16))
    with pytest.raises(ValueError, match="grad"):
        B.grad_quant(d, act.to(torch.bfloat16), codes, scales)
    with pytest.raises(ValueError, match="seen"):
        B.encode_seen(d, act, ids, m, torch.zeros(4, dtype=torch.uint8), 1, torch.zeros(2, dtype=torch.int32),
                      codes, scales)
    with pytest.raises(ValueError, match="first"):
        B.encode_seen(d, act, ids, m, torch.zeros(4, dtype=torch.int32), 1, torch.zeros(3, dtype=torch.int32),
                      codes, scales)
    with pytest.raises(ValueError, match="sample_ids"):
        B.encode_job(d, act, ids.to(torch.int32), m, codes, scales)
    # well-formed arguments pass the checks and reach the library (null pointers: refused there)
    with pytest.raises(B.AqsgdError) as e:
        B.encode(d, act, ids, m, codes, scales, stream=type("S", (), {"cuda_stream": 0})())
    assert e.value.status == -1


def test_job_layout_matches_header():
    assert ctypes.sizeof(B.Job) == 8 + 48 + 9 * 8 + 8
    assert B.Job.desc.offset == 8 and B.Job.src.offset == 56 and B.Job.out.offset == 96


def test_header_is_plain_c_and_a_c_client_links(tmp_path):
    """The boundary is a C ABI: the header compiles as C99 on its own, and a C program
    that only knows the header links against the library and reads a size through it."""
    import ctypes.util
    import shutil
    import subprocess
    from pathlib import Path
    root = Path(__file__).resolve().parent.parent
    header = root / "include" / "aqsgd.h"
    gcc = shutil.which("gcc")
    assert gcc, "gcc is part of the image"
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-pedantic", "-Werror", "-fsyntax-only", "-x", "c",
                    str(header)], check=True)
    lib = root / "paper_2206_01299_amd" / "libaqsgd.so"
    src = tmp_path / "client.c"
    src.write_text('#include <stdio.h>\n#include "aqsgd.h"\n'
                   'int main(void) {\n'
                   '    aqsgd_desc d = {4, 1638400, 8192, 4, 1600, AQSGD_F16, AQSGD_ROUND_NEAREST, 0};\n'
                   '    printf("%zu %zu %zu %s\\n", aqsgd_codes_bytes(&d), aqsgd_scales_count(&d), sizeof(aqsgd_job),\n'
                   '           aqsgd_strerror(-3));\n'
                   '    return aqsgd_encode(&d, NULL, NULL, NULL, NULL, NULL, NULL) == AQSGD_ERR_NULL ? 0 : 1;\n'
                   '}\n')
    exe = tmp_path / "client"
    subprocess.run([gcc, "-std=c99", f"-I{header.parent}", str(src), str(lib), f"-Wl,-rpath,{lib.parent}",
                    "-Wl,-rpath,/opt/rocm/lib", "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split(maxsplit=3)
    assert out[0] == str(4 * 1638400 * 4 // 8) and out[1] == str(4 * 1638400 // 1600)
    assert int(out[2]) == ctypes.sizeof(B.Job)           # the binding's mirror of aqsgd_job has the C size
    assert "group" in out[3]
