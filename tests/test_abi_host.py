"""The C-ABI library on a host without a GPU: it loads, exports every function the header declares, and its
argument validation (which runs before any HIP call) returns the documented codes.  No compute calls."""
import ctypes as C
import os
import re
import subprocess

import pytest

from paper_2509_16434_amd import configs, learner as L

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "ppo_learner.h")
DIAG_HEADER = os.path.join(ROOT, "include", "ppo_learner_diag.h")   # tracing / diagnostic aids, not the learner's path


def _declared(headers=(HEADER, DIAG_HEADER)):
    names = []
    for h in headers:
        text = re.sub(r"/\*.*?\*/", "", open(h).read(), flags=re.S)
        names += re.findall(r"^(?:int|int64_t|const char\*)\s+(\w+)\s*\(", text, flags=re.M)
    return names


def test_library_exports_every_declared_function():
    names = _declared()
    assert len(names) >= 20 and len(set(names)) == len(names)
    lib = C.CDLL(L.LIB_PATH)
    for n in names:
        assert hasattr(lib, n), n
    # the binding marshals exactly the declared functions
    assert sorted(L.EXPORTS) == sorted(names)


def test_the_four_path_entry_points_are_declared():
    names = set(_declared((HEADER,)))
    assert {"ppo_buffer_write", "ppo_gae", "ppo_update", "distill_update"} <= names
    assert set(_declared((DIAG_HEADER,))) == {"ppo_profile", "ppo_profile_report", "ppo_diag_gemm", "ppo_diag_peak"}


def text_of_desc():
    text = open(HEADER).read()
    return text[text.index("int32_t num_envs, horizon;"):text.index("} ppo_net_desc;")]


def test_struct_sizes_match_the_header_layout():
    # ppo_hparams: 15 floats, 5 int32, one uint64; ppo_mb_stats: 7 floats, int32, float
    assert C.sizeof(L.HParams) == 15 * 4 + 5 * 4 + 8 and L.HParams.seed.offset == 80
    assert C.sizeof(L.MbStats) == 36 and L.MbStats.lr.offset == 32
    # ppo_net_desc: 9 + 1 + 8 + 3 + 1 + 8 + 2 + 6 int32 fields, in the header's order
    assert C.sizeof(L.NetDesc) == 4 * (9 + 1 + 8 + 3 + 1 + 8 + 2 + 6)
    dbody = re.sub(r"/\*.*?\*/", "", text_of_desc(), flags=re.S)
    dnames = [n for n in re.findall(r"(\w+)(?:\[\w+\])?\s*[,;]", dbody)]
    assert dnames == [f for f, _ in L.NetDesc._fields_]
    text = open(HEADER).read()
    body = text[text.index("float gamma, lambda;"):text.index("} ppo_hparams;")]
    body = re.sub(r"/\*.*?\*/", "", body, flags=re.S)
    names = re.findall(r"(\w+)\s*[,;]", body)
    assert names == [("lambda" if f == "lam" else f) for f, _ in L.HParams._fields_]


def test_header_is_plain_c(tmp_path):
    for h in (HEADER, DIAG_HEADER):
        text = open(h).read()
        assert 'extern "C"' in text and "torch" not in text and "std::" not in text
    # both headers compile as C99 and as C++, on their own, with every warning an error
    src = tmp_path / "use.c"
    src.write_text('#include "ppo_learner_diag.h"\nint main(void) { ppo_hparams hp; ppo_net_desc d; ppo_mb_stats s; (void)hp; (void)d; (void)s;'
                   ' return PPO_STATIC_PERM_MAX > 0 && PPO_OK == 0 ? 0 : 1; }\n')
    inc = os.path.join(ROOT, "include")
    subprocess.check_call(["gcc", "-std=c99", "-pedantic", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-I", inc, str(src)])
    subprocess.check_call(["g++", "-std=c++17", "-Wall", "-Wextra", "-Werror", "-fsyntax-only", "-x", "c++", "-I", inc, str(src)])


def test_static_permutation_validates_before_touching_the_gpu():
    lib = L._lib
    assert lib.ppo_permutation_static(-1, 1, 1, 1, None, None) == L.PPO_EINVAL
    assert lib.ppo_permutation_static(L.STATIC_PERM_MAX + 1, 1, 1, 1, None, None) == L.PPO_ESHAPE
    assert b"at most" in lib.ppo_last_error(None)
    assert lib.ppo_permutation_static(0, 1, 1, 1, None, None) == L.PPO_OK
    assert lib.ppo_permutation_static(16, 1, 1, 1, None, None) == L.PPO_EINVAL   # d_perm is NULL
    text = open(HEADER).read()
    assert "#define PPO_STATIC_PERM_MAX (1 << 20)" in text and L.STATIC_PERM_MAX == 1 << 20


@pytest.mark.parametrize("change,code", [
    (dict(conv_k=5), L.PPO_ESHAPE), (dict(conv_stride=1), L.PPO_ESHAPE), (dict(conv_pad=0), L.PPO_ESHAPE),
    (dict(proprio_dim=3), L.PPO_ESHAPE), (dict(act_dim=40), L.PPO_ESHAPE), (dict(act_dim=0), L.PPO_ESHAPE),
    (dict(fc_dim=[12]), L.PPO_ESHAPE), (dict(fc_dim=[]), L.PPO_ESHAPE), (dict(conv_ch=[12]), L.PPO_ESHAPE),
    (dict(in_h=0), L.PPO_ESHAPE), (dict(has_value_head=2), L.PPO_EINVAL),
    (dict(aux_hidden=12, aux_dim=2), L.PPO_ESHAPE), (dict(aux_hidden=16, aux_dim=2), L.PPO_ESHAPE),   # the second: an actor-critic
    (dict(has_value_head=0, aux_hidden=16, aux_dim=12), L.PPO_ESHAPE), (dict(has_value_head=0, aux_hidden=16, aux_dim=0), L.PPO_ESHAPE),
    (dict(layer_norm=2), L.PPO_EINVAL), (dict(embed_dim=12), L.PPO_ESHAPE), (dict(lstm_layers=5, lstm_units=16), L.PPO_ESHAPE),
    (dict(lstm_layers=1, lstm_units=12), L.PPO_ESHAPE), (dict(has_value_head=0, lstm_layers=1, lstm_units=16), L.PPO_ESHAPE),
])
def test_create_rejects_bad_geometry_before_touching_the_gpu(change, code):
    net = dict(configs.get_config(0)["net"], **change)
    with pytest.raises(L.LearnerError) as e:
        L.Learner(net, 8, 2, "fp32")
    assert e.value.code == code, str(e.value)
    assert len(str(e.value)) > 10


def test_create_rejects_bad_sizes():
    net = configs.get_config(0)["net"]
    for n, t in ((0, 2), (8, 0), (-1, 2)):
        with pytest.raises(L.LearnerError) as e:
            L.Learner(net, n, t, "fp32")
        assert e.value.code in (L.PPO_ESHAPE, L.PPO_EINVAL)
    with pytest.raises(L.LearnerError) as e:
        L.Learner(net, 8, 2, "fp32", max_chunk=-5)
    assert e.value.code == L.PPO_EINVAL


def test_null_handles_are_einval_not_a_crash():
    lib = L._lib
    assert lib.ppo_create(None, None, None) == L.PPO_EINVAL
    assert lib.ppo_destroy(None) == L.PPO_EINVAL
    assert lib.ppo_gae(None, None, C.c_float(0.9), C.c_float(0.9)) == L.PPO_EINVAL
    assert lib.ppo_update(None, None, None) == L.PPO_EINVAL
    assert lib.distill_update(None, None, None) == L.PPO_EINVAL
    assert lib.ppo_buffer_write(None, 0, None, None, None, None, None, None, None) == L.PPO_EINVAL
    assert lib.ppo_buffer_write_range(None, 0, 0, 1, None, None, None, None, None, None, None) == L.PPO_EINVAL
    assert lib.ppo_act(None, 0, None, None, None, None, None, None) == L.PPO_EINVAL
    assert lib.ppo_buffer_write_outcome(None, 0, None, None) == L.PPO_EINVAL
    assert lib.ppo_param_count(None) < 0
    assert lib.ppo_diag_gemm(4, 4, 7, None, None, None) == L.PPO_EINVAL
    import ctypes
    r = ctypes.c_float()
    assert lib.ppo_diag_peak(6, 1 << 20, 1, ctypes.byref(r)) == L.PPO_EINVAL    # no such kind
    assert lib.ppo_diag_peak(5, 9, 1, ctypes.byref(r)) == L.PPO_EINVAL          # at most 8 vector instructions per MFMA
    assert lib.ppo_diag_peak(0, 100, 1, ctypes.byref(r)) == L.PPO_EINVAL        # a copy needs at least 1 MiB
    assert lib.ppo_diag_peak(4, 0, 1, None) == L.PPO_EINVAL
    assert lib.ppo_get_adaptive_lr(None, None, None) == L.PPO_EINVAL
    assert lib.ppo_set_adaptive_lr(None, 1e-3, 1) == L.PPO_EINVAL


def test_binding_refuses_host_tensors():
    import torch
    with pytest.raises(ValueError):
        L._dev(torch.zeros(4))
    with pytest.raises(ValueError):
        L._dev(torch.zeros(4, device="meta") if False else torch.zeros(2, 2).t())
