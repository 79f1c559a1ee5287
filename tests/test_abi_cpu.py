"""Host-side checks of the C ABI that need no GPU: the library loads, exports every symbol the
header declares, sizes and validates configurations."""
import ctypes
import os
import re

import pytest

from paper_2011_13635_amd import binding, synth


def declared_symbols(repo_root):
    text = open(os.path.join(repo_root, "include", "mslt.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(mslt_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol(repo_root):
    lib = binding.load_library()
    names = declared_symbols(repo_root)
    assert len(names) >= 15
    assert sorted(binding.EXPORTS) == names
    for n in names:
        assert getattr(lib, n) is not None


def test_query_sizes_scale_with_config():
    tiny = binding.mslt_query_sizes(binding.make_config(synth.tiny_shape(), 4, 64, 0))
    base = binding.mslt_query_sizes(binding.make_config(synth.bert_base_shape(), 64, 128, 1))
    assert all(b > t > 0 for b, t in zip(base, tiny))
    p, g, o, w = base
    assert p == g and o == 2 * p
    # 12-layer Base with head: about 110 M parameters in fp32 (+ padding of the vocabulary to 128 rows)
    assert 109e6 * 4 < p < 111e6 * 4
    assert p % 256 == 0 and w % 256 == 0


def test_workspace_follows_the_number_of_layers_that_can_train():
    # Section 3.2: the bottom layers only take part in the forward computation, so the per-layer stash of
    # activations is needed for max_trainable_layers layers only (0 = every layer); parameters, gradients and
    # moments do not depend on it
    sh = synth.bert_large_shape(24)
    full = binding.mslt_query_sizes(binding.make_config(sh, 32, 512, 1))
    six = binding.mslt_query_sizes(binding.make_config(sh, 32, 512, 1, max_trainable_layers=6))
    twelve = binding.mslt_query_sizes(binding.make_config(sh, 32, 512, 1, max_trainable_layers=12))
    assert full[:3] == six[:3] == twelve[:3]
    assert six[3] < twelve[3] < full[3]
    # the stash of one layer is the same size whichever range it comes from
    assert abs((full[3] - twelve[3]) / 12 - (twelve[3] - six[3]) / 6) < 0.01 * (twelve[3] - six[3]) / 6
    assert binding.mslt_query_sizes(binding.make_config(sh, 32, 512, 1, max_trainable_layers=24)) == full
    cfg = binding.make_config(sh, 32, 512, 1)
    cfg.max_trainable_layers = -1
    with pytest.raises(binding.MsltError):
        binding.mslt_query_sizes(cfg)


@pytest.mark.parametrize("field,value", [("hidden", 130), ("hidden", 4096), ("n_heads", 5), ("precision", 2),
                                         ("type_vocab", 9), ("max_seq", 1024), ("n_layers_max", 0), ("vocab", 1)])
def test_bad_config_is_rejected(field, value):
    cfg = binding.make_config(synth.tiny_shape(), 4, 64, 0)
    setattr(cfg, field, value)
    with pytest.raises(binding.MsltError) as ei:
        binding.mslt_query_sizes(cfg)
    assert ei.value.code == binding.MSLT_ERR_ARG
    assert "config" in str(ei.value)


def test_null_arguments_return_error_codes():
    lib = binding.load_library()
    assert lib.mslt_query_sizes(None, None, None, None, None) == binding.MSLT_ERR_ARG
    assert lib.mslt_stage_step(None, 0, 1, 0, None, None) == binding.MSLT_ERR_ARG
    assert lib.mslt_apply_update(None, None) == binding.MSLT_ERR_ARG
    assert lib.mslt_get_grads(None, None, 0) == binding.MSLT_ERR_ARG
    assert lib.mslt_load_params(None, None, 0) == binding.MSLT_ERR_ARG
    assert lib.mslt_destroy(None) == 0
    cfg = binding.make_config(synth.tiny_shape(), 4, 64, 0)
    h = ctypes.c_void_p()
    # null arenas are refused before any GPU call
    assert lib.mslt_init_model(ctypes.byref(cfg), None, None, None, None, None, ctypes.byref(h)) == binding.MSLT_ERR_ARG
    assert b"null" in lib.mslt_last_error()


def test_model_needs_a_gpu():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(RuntimeError):
        binding.Model(binding.make_config(synth.tiny_shape(), 4, 64, 0))


def test_ctypes_structs_match_the_header_layout(tmp_path, repo_root):
    """sizeof and every field offset of the C structs, as gcc lays them out from include/mslt.h, against the
    ctypes mirrors of the binding (a reordered or missing field would silently corrupt every call)."""
    import ctypes
    import shutil
    import subprocess
    if shutil.which("gcc") is None:
        pytest.skip("no C compiler")
    structs = {"mslt_config": binding.Config, "mslt_batch": binding.Batch, "mslt_opt": binding.Opt,
               "mslt_tensor_desc": binding.TensorDesc, "mslt_profile_entry": binding.ProfileEntry}
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "mslt.h"', 'int main(void) {']
    for cname, cls in structs.items():
        lines.append(f'  printf("{cname} size %zu\\n", sizeof({cname}));')
        for fname, _ in cls._fields_:
            lines.append(f'  printf("{cname} {fname} %zu\\n", offsetof({cname}, {fname}));')
    lines += ['  return 0;', '}']
    src = tmp_path / "layout.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "layout"
    subprocess.run(["gcc", "-std=c99", "-I", os.path.join(repo_root, "include"), str(src), "-o", str(exe)], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split("\n")
    seen = 0
    for line in out:
        if not line:
            continue
        cname, fname, value = line.split()
        cls = structs[cname]
        want = ctypes.sizeof(cls) if fname == "size" else getattr(cls, fname).offset
        assert int(value) == want, (cname, fname, value, want)
        seen += 1
    assert seen == sum(len(c._fields_) + 1 for c in structs.values())
