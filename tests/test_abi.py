"""The C-ABI library loads and exports every function include/sjd.h declares (no GPU needed)."""
import ctypes
import os
import re

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    src = open(os.path.join(ROOT, "include", "sjd.h")).read()
    src = re.sub(r"/\*.*?\*/", "", src, flags=re.S)
    return sorted(set(re.findall(r"\b(sjd_[a-z_0-9]+)\s*\(", src)))


def test_header_declares_the_path():
    names = _declared()
    for must in ("sjd_init_model", "sjd_prefill", "sjd_step", "sjd_generate"):
        assert must in names


def test_library_exports_every_declared_symbol():
    from paper_2410_01699_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name
    assert sorted(binding.EXPORTS) == _declared()


def test_error_strings_and_argument_checks_without_gpu():
    from paper_2410_01699_amd import binding
    assert binding.sjd_strerror(0) == "ok"
    assert "invalid" in binding.sjd_strerror(binding.SJD_EINVAL)
    # null / malformed arguments are rejected before any HIP call
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.sjd_init_model.restype = ctypes.c_int
    out = ctypes.c_void_p()
    assert lib.sjd_init_model(None, None, ctypes.c_size_t(0), ctypes.byref(out)) == binding.SJD_EINVAL
    cfg = binding.sjd_config(2, 130, 4, 512, 1024, 0, 1024, 64, 0, 10000.0, 1e-5)     # d % heads != 0
    assert lib.sjd_init_model(ctypes.byref(cfg), None, ctypes.c_size_t(0), ctypes.byref(out)) == binding.SJD_EINVAL
    assert lib.sjd_kv_create(None, ctypes.byref(out)) == binding.SJD_EINVAL
    assert lib.sjd_step(None, None, None, None, 4, None, None, 0, 0, 0, None, None, None, None) == binding.SJD_EINVAL


def test_bench_refuses_more_than_one_gpu():
    """one GPU only: asking for more exits with a message instead of launching anything"""
    import subprocess, sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr


def test_null_arguments_of_the_wider_entry_points_without_gpu():
    from paper_2410_01699_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    E = binding.SJD_EINVAL
    assert lib.sjd_prefill_uncond(None, None, None, 0, None, 0, ctypes.c_float(3.0), None, None, None, None) == E
    assert lib.sjd_decode_steps_batch(None, None, 2, 1, None) == E
    assert lib.sjd_generate_batch(None, None, 2, None, None, None, None, 8, 4, None, None, None, None, None) == E
    assert lib.sjd_forward_logits_batch(None, None, 2, None, 4, None, None) == E
    assert lib.sjd_profile_steps_batch(None, None, 2, 1, None, None) == E
    assert lib.sjd_generate_cfg(None, None, None, 0, None, 0, None, 0, None, 0, ctypes.c_float(3.0), 8, 4, None, None,
                                ctypes.c_uint64(0), None, None) == E


def test_static_verify_checks_its_arguments_and_its_limit_without_gpu():
    """the entry point that allocates nothing rejects null pointers and sizes beyond its static scratch
    before it touches the GPU"""
    from paper_2410_01699_amd import binding
    lib = ctypes.CDLL(binding.LIB_PATH)
    lib.sjd_strerror.restype = ctypes.c_char_p
    u64 = ctypes.c_uint64
    assert lib.sjd_verify_static(None, None, None, 4, 64, 0, None, None, 0, None, None, u64(0), u64(0), None, None, None,
                                 None) == binding.SJD_EINVAL
    dummy = (ctypes.c_float * 4)()           # never dereferenced: the size check comes first
    p = ctypes.cast(dummy, ctypes.c_void_p)
    smp, init = binding.sjd_sampler(10, 1.0), binding.sjd_init(0, 0, -1, 0)
    L, V = 32, 16384
    assert (L + 1) * V > binding.SJD_STATIC_VERIFY_FLOATS
    rc = lib.sjd_verify_static(p, p, p, L, V, 0, ctypes.byref(smp), ctypes.byref(init), 0, None, None, u64(1), u64(1), p, p, p,
                               None)
    assert rc == binding.SJD_ELIMIT
    assert b"static scratch" in lib.sjd_strerror(rc)


def test_binding_constants_equal_the_header():
    """limits and error codes are typed twice (C header, Python binding): they must agree"""
    from paper_2410_01699_amd import binding
    src = open(os.path.join(ROOT, "include", "sjd.h")).read()

    def define(name):
        m = re.search(r"#define\s+" + name + r"\s+\(?([^)\n/]+)\)?", src)
        assert m, name
        return int(eval(m.group(1).strip(), {"__builtins__": {}}))          # plain integer expressions only

    for name in ("SJD_OK", "SJD_EINVAL", "SJD_ENOMEM", "SJD_ESEQ", "SJD_EHIP", "SJD_ELIMIT", "SJD_MAX_WINDOW", "SJD_MAX_ROWS",
                 "SJD_STATIC_VERIFY_FLOATS", "SJD_MAX_SAMP_VOCAB"):
        assert define(name) == getattr(binding, name), name
