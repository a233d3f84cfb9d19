"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the
header declares, and rejects bad arguments / call orders before launching anything."""
import ctypes
import os
import re

import pytest

from paper_2310_01801_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(binding.LIB_PATH):
        from paper_2310_01801_amd import build
        build.build(verbose=False)
    return binding.load_library()


def test_every_declared_symbol_is_exported(lib):
    header = open(os.path.join(ROOT, "include", "fastgen.h")).read()
    declared = set(re.findall(r"\b(fastgen_[a-z_]+)\s*\(", header))
    declared.discard("fastgen_ctx")
    assert declared == set(binding.EXPORTED)
    for name in declared:
        assert getattr(lib, name) is not None
    assert b"gfx950" in lib.fastgen_version()


def test_config_struct_matches_header():
    # field order/types of the ctypes mirror against the C declaration
    header = open(os.path.join(ROOT, "include", "fastgen.h")).read()
    body = header[header.index("typedef struct {"):header.index("} fg_config;")]
    names = re.findall(r"^\s*(?:int32_t|int64_t|double|float)\s+([A-Za-z_]+(?:\s*,\s*[A-Za-z_]+)*)(?:\[\d+\])?\s*;", body, re.M)
    flat = [x.strip() for grp in names for x in grp.split(",")]
    assert flat == [f[0] for f in binding.FgConfig._fields_]


def _cfg(**kw):
    base = dict(num_units=8, num_seqs=2, head_dim=128, dtype=binding.torch.bfloat16, prompt_len=64,
                max_new_tokens=4, T=0.95, r_l=0.3, r_f=0.3)
    base.update(kw)
    return binding.make_config(**base)


def test_workspace_bytes_and_validation(lib):
    good = _cfg()
    nbytes = binding.fastgen_workspace_bytes(good)
    assert nbytes > 8 * 68 * 128 * 2 * 2 and nbytes % 256 == 0
    assert binding.fastgen_workspace_bytes(_cfg(cache_tokens=100)) < nbytes
    assert binding.fastgen_workspace_bytes(_cfg(family=(8, 4, 12, 0), forced_policy=2)) == nbytes
    assert binding.fastgen_workspace_bytes(_cfg(group_size=4)) > nbytes   # per-head lse, logits, partials
    assert binding.fastgen_workspace_bytes(_cfg(group_size=0)) == nbytes
    # the accepted maximum: 131072 tokens per unit, 16 query heads per K/V head, float32
    big = _cfg(num_units=2, num_seqs=1, prompt_len=131000, max_new_tokens=72, group_size=16, dtype=binding.torch.float32)
    assert binding.fastgen_workspace_bytes(big) > 2 * 131072 * 128 * 4 * 2
    for bad in (dict(head_dim=96), dict(num_seqs=3), dict(T=0.0), dict(T=1.5), dict(r_l=-0.1),
                dict(prompt_len=0), dict(forced_policy=7), dict(num_units=0), dict(family=(1, 16, 0, 0)),
                dict(family=(1, 0, 0, 8), forced_policy=1), dict(group_size=17), dict(group_size=-1),
                # beyond what the kernels' 32-bit row offsets and the read-back bitmap cover
                dict(prompt_len=131073, max_new_tokens=0), dict(prompt_len=131072, max_new_tokens=1),
                dict(prompt_len=1 << 20), dict(max_new_tokens=1 << 20), dict(prompt_len=70000, max_new_tokens=70000),
                # more work items than a 32-bit grid holds
                dict(num_units=1 << 24, num_seqs=1, prompt_len=131072, max_new_tokens=0)):
        assert binding.fastgen_workspace_bytes(_cfg(**bad)) == 0, bad


def test_create_and_call_order_errors_without_launching(lib):
    cfg = _cfg()
    nbytes = binding.fastgen_workspace_bytes(cfg)
    ctx = ctypes.c_void_p()
    fake = ctypes.c_void_p(0x10000)  # never dereferenced: every call below fails on the host
    assert lib.fastgen_create(ctypes.byref(cfg), None, nbytes, ctypes.byref(ctx)) == binding.FG_EINVAL
    assert lib.fastgen_create(ctypes.byref(cfg), ctypes.c_void_p(0x10008), nbytes, ctypes.byref(ctx)) == binding.FG_EINVAL
    assert lib.fastgen_create(ctypes.byref(cfg), fake, nbytes - 1, ctypes.byref(ctx)) == binding.FG_ENOMEM
    assert lib.fastgen_create(ctypes.byref(cfg), fake, nbytes, ctypes.byref(ctx)) == binding.FG_OK
    assert lib.fastgen_profile(ctx, None, None, None, None, None, None, None, None) == binding.FG_EINVAL
    assert b"required" in lib.fastgen_last_error(ctx)
    assert lib.fastgen_profile(ctx, 0x10004, 0x10000, 0x10000, None, None, None, None, None) == binding.FG_EINVAL
    assert lib.fastgen_compact(ctx, 0x10000, 0x10000, None) == binding.FG_ESTATE
    assert lib.fastgen_decode_step(ctx, 0x10000, 0x10000, 0x10000, 0x10000, 0x10000, None) == binding.FG_ESTATE
    assert lib.fastgen_export_state(ctx, None, None, None, None, None, None, None, None) == binding.FG_ESTATE
    assert lib.fastgen_destroy(ctx) == binding.FG_OK
    assert lib.fastgen_destroy(None) == binding.FG_OK


def test_static_profile_rejects_bad_arguments_on_the_host(lib):
    fake = 0x10000  # never dereferenced: every call below fails before anything is launched
    cfg = _cfg()
    call = lib.fastgen_profile_static
    assert call(None, fake, fake, fake, None, None, None, None, None) == binding.FG_EINVAL
    assert b"config is NULL" in lib.fastgen_last_error(None)
    assert call(ctypes.byref(_cfg(head_dim=96)), fake, fake, fake, None, None, None, None, None) == binding.FG_EINVAL
    assert call(ctypes.byref(cfg), None, fake, fake, None, None, None, None, None) == binding.FG_EINVAL
    assert call(ctypes.byref(cfg), fake + 4, fake, fake, None, None, None, None, None) == binding.FG_EINVAL
    assert b"16-byte aligned" in lib.fastgen_last_error(None)
    # beyond the static scratch array (32 MiB): refused with the sizes in the message
    big = _cfg(num_units=1024, num_seqs=1, prompt_len=2048)
    assert call(ctypes.byref(big), fake, fake, fake, None, None, None, None, None) == binding.FG_ENOMEM
    assert b"static array holds 33554432" in lib.fastgen_last_error(None)


def test_classify_rejects_bad_arguments_on_the_host(lib):
    fake = 0x10000
    ids = (ctypes.c_int32 * 70)(*range(70))
    call = lib.fastgen_classify
    assert call(None, 0, None, 0, None, 0, None, None) == binding.FG_OK            # nothing to do
    assert call(None, 8, None, 0, None, 0, fake, None) == binding.FG_EINVAL
    assert call(fake, 8, None, 0, None, 0, None, None) == binding.FG_EINVAL
    assert call(fake, -1, None, 0, None, 0, fake, None) == binding.FG_EINVAL
    assert call(fake, 8, ids, 65, None, 0, fake, None) == binding.FG_EINVAL        # more than 64 ids
    assert b"at most 64" in lib.fastgen_last_error(None)
    assert call(fake, 8, None, 3, None, 0, fake, None) == binding.FG_EINVAL        # a count without a list


def test_microbenchmark_library_loads_and_rejects_bad_arguments(lib):
    # the measurement aid of bench.py: built next to the main library, one C entry point
    path = os.path.join(os.path.dirname(binding.LIB_PATH), "libfgubench.so")
    assert os.path.exists(path), "python -m paper_2310_01801_amd.build builds it"
    ub = ctypes.CDLL(path)
    ub.fg_ubench_run.restype = ctypes.c_int
    ub.fg_ubench_run.argtypes = [ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p,
                                 ctypes.c_void_p, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    ns, mhz = ctypes.c_double(), ctypes.c_double()
    assert ub.fg_ubench_run(0, 1, 1, 0x10000, None, None, ctypes.byref(ns), None) == -1      # mode out of range
    assert ub.fg_ubench_run(1, 0, 1, 0x10000, None, None, ctypes.byref(ns), None) == -1
    assert ub.fg_ubench_run(1, 1, 1, None, None, None, ctypes.byref(ns), None) == -1
    assert ub.fg_ubench_run(1, 1, 1, 0x10000, None, None, ctypes.byref(ns), ctypes.byref(mhz)) == -1  # clock without its buffer
