"""The C-ABI library loads, exports every symbol include/eet.h declares, and rejects bad
arguments before any device work (no GPU needed: these paths return before the first HIP call)."""
import ctypes as C
import os
import re

import pytest

from oracle import eet_oracle as orc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HEADER = os.path.join(ROOT, "include", "eet.h")


@pytest.fixture(scope="module")
def eet():
    from paper_2104_12470_amd import eet as binding
    if not os.path.exists(binding.LIB_PATH):
        from paper_2104_12470_amd.build import build_library
        build_library(verbose=False)
    binding.lib()
    return binding


def declared_functions():
    text = re.sub(r"/\*.*?\*/", "", open(HEADER).read(), flags=re.S)
    return sorted(set(re.findall(r"\b(eet_[a-z0-9_]+)\s*\(", text)))


def test_every_declared_symbol_is_exported(eet):
    names = declared_functions()
    assert "eet_layer_create" in names and "eet_prefill" in names and "eet_decode_step" in names \
        and "eet_layer_destroy" in names
    for n in names:
        assert hasattr(eet.lib(), n), f"{n} declared in eet.h but not exported"
    assert sorted(eet.EXPORTS) == names            # the binding covers the whole header


def test_size_queries(eet):
    cfg = eet.make_config(1024, 16, 4096, 8, 512, 1024)
    # Section 3.1: 2*b*h*s elements per layer, fp16
    assert eet.eet_kv_cache_bytes(cfg) == 2 * orc.kv_cache_elements(8, 1024, 1024, 1)
    ws = eet.eet_workspace_bytes(cfg)
    T = 8 * 512
    need = 2 * T * (3 * 1024 + 4096)               # three [T,H] buffers and one [T,F] buffer, fp16
    assert need <= ws <= need + (1 << 20)
    # same order as the paper's activation-cache + buffer bound (Sections 3.1, 3.2), in bytes
    bound = 2 * (orc.activation_cache_elements(8, 1024, 512) + orc.buffer_elements(8, 512, 1024, 16))
    assert ws <= bound
    assert eet.eet_workspace_bytes(eet.make_config(96, 1, 256, 1, 8, 8)) == 0          # head size 96
    assert eet.eet_kv_cache_bytes(eet.make_config(0, 1, 256, 1, 8, 8)) == 0


def _fake_layer(eet, cfg):
    w = eet.LayerWeights(*[0x10000 + 0x100 * i for i in range(12)])
    h = C.c_void_p()
    rc = eet.lib().eet_layer_create(C.byref(cfg), C.byref(w), 0x100000, C.byref(h))
    return rc, h


def test_create_rejects_bad_configs(eet):
    L = eet.lib()
    rc, h = _fake_layer(eet, eet.make_config(768, 12, 3072, 4, 64, 64))
    assert rc == eet.EET_OK and h.value
    assert L.eet_layer_destroy(h) == eet.EET_OK
    for cfg, code in [(eet.make_config(768, 5, 3072, 4, 64, 64), eet.EET_ERR_INVALID_ARG),       # heads !| hidden
                      (eet.make_config(960, 10, 3072, 4, 64, 64), eet.EET_ERR_UNSUPPORTED_SHAPE),  # d = 96
                      (eet.make_config(768, 12, 3000, 4, 64, 64), eet.EET_ERR_UNSUPPORTED_SHAPE),  # ffn % 64
                      (eet.make_config(768, 12, 3072, 129, 64, 64), eet.EET_ERR_UNSUPPORTED_SHAPE),
                      (eet.make_config(768, 12, 3072, 4, 64, 32), eet.EET_ERR_UNSUPPORTED_SHAPE),  # s < p
                      (eet.make_config(768, 12, 3072, 0, 64, 64), eet.EET_ERR_INVALID_ARG)]:
        rc, h = _fake_layer(eet, cfg)
        assert rc == code and not h.value
        assert L.eet_last_error()
    w = eet.LayerWeights(*[0x10000] * 11, 0)
    h = C.c_void_p()
    cfg = eet.make_config(768, 12, 3072, 4, 64, 64)
    assert L.eet_layer_create(C.byref(cfg), C.byref(w), 0x100000, C.byref(h)) == eet.EET_ERR_INVALID_ARG
    assert L.eet_layer_create(C.byref(cfg), C.byref(eet.LayerWeights(*[0x10000] * 12)), 0x100010, C.byref(h)) \
        == eet.EET_ERR_INVALID_ARG                                                              # workspace alignment


def test_prefill_and_decode_validate_before_any_launch(eet):
    L = eet.lib()
    cfg = eet.make_config(768, 12, 3072, 4, 64, 80)
    rc, h = _fake_layer(eet, cfg)
    assert rc == 0
    lens = (C.c_int32 * 4)(5, 2, 4, 10)
    P = 0x200000
    assert L.eet_decode_step(h, P, P, P, None) == eet.EET_ERR_STATE                  # decode before prefill
    assert b"prefill" in L.eet_last_error()
    assert L.eet_cache_lens(h, lens, None) == eet.EET_ERR_STATE
    assert L.eet_prefill(h, lens, 5, 10, P, P, P, None) == eet.EET_ERR_CAPACITY      # batch > max_batch
    assert L.eet_prefill(h, lens, 4, 65, P, P, P, None) == eet.EET_ERR_CAPACITY      # padded_len > max_prompt
    assert L.eet_prefill(h, lens, 4, 9, P, P, P, None) == eet.EET_ERR_INVALID_ARG    # q_lens[3] = 10 > 9
    assert L.eet_prefill(h, (C.c_int32 * 4)(5, 0, 4, 10), 4, 10, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_prefill(h, lens, 0, 10, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_prefill(h, lens, 4, 10, None, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_prefill(h, lens, 4, 10, P + 2, P, P, None) == eet.EET_ERR_INVALID_ARG   # alignment
    assert L.eet_decode_step(h, P, P, P, None) == eet.EET_ERR_STATE                  # failures changed no state
    assert L.eet_restore(h, None, 4, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_restore(h, lens, 5, None) == eet.EET_ERR_CAPACITY                   # batch > max_batch
    assert L.eet_restore(h, (C.c_int32 * 4)(5, 2, 4, 81), 4, None) == eet.EET_ERR_INVALID_ARG   # 81 > max_seq 80
    assert L.eet_restore(h, (C.c_int32 * 4)(5, 0, 4, 10), 4, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_restore(None, lens, 4, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_stack_restore(None, lens, 4, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_decode_step(h, P, P, P, None) == eet.EET_ERR_STATE                  # ... still none
    assert L.eet_layer_destroy(h) == 0


def test_op_entry_points_validate(eet):
    L = eet.lib()
    P = 0x200000
    lens = (C.c_int32 * 2)(3, 9)
    assert L.eet_op_layernorm(None, P, P, P, 4, 64, 1e-5, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_layernorm(P, P, P, P, 4, 0, 1e-5, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_softmax_maskfree(P, lens, 2, 2, 8, 1.0, None) == eet.EET_ERR_INVALID_ARG   # len 9 > S 8
    assert L.eet_op_softmax_maskfree(P, lens, 200, 2, 16, 1.0, None) == eet.EET_ERR_CAPACITY
    assert L.eet_op_softmax_maskfree_left_padded(P, lens, 2, 2, 8, 1.0, None) == eet.EET_ERR_INVALID_ARG   # len 9 > S 8
    assert L.eet_op_softmax_maskfree_left_padded(None, lens, 2, 2, 16, 1.0, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_bias_gelu(P, None, P, 4, 64, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_bias_residual(P, P, None, P, 4, 64, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_linear(P, P, P, None, P, 4, 100, 64, 0, None) == eet.EET_ERR_UNSUPPORTED_SHAPE
    assert L.eet_op_linear(P, P, P, P, P, 4, 64, 64, 1, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_attention_prefill(P, P, P, P, lens, 2, 16, 2, 96, 16, None) == eet.EET_ERR_UNSUPPORTED_SHAPE
    assert L.eet_op_attention_prefill(P, P, P, P, lens, 2, 16, 2, 64, 8, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_attention_decode(P, P, P, P, P, 2, 2, 64, 16, None, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_attention_decode_scratch_bytes(2, 2, 64, 4096) > 0
    # unfused form: needs a buffer manager, a padded length that is a multiple of 8, and an arena that holds the scores
    mgr = C.c_void_p()
    assert L.eet_bufmgr_create(0x7F0000000000, 1024, C.byref(mgr)) == eet.EET_OK
    lens8 = (C.c_int32 * 2)(3, 8)
    assert L.eet_op_attention_unfused(P, P, P, P, lens8, 2, 16, 2, 64, 16, None, 0, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_attention_unfused(P, P, P, P, lens8, 2, 12, 2, 64, 16, mgr, 0, None) == eet.EET_ERR_UNSUPPORTED_SHAPE
    assert L.eet_op_attention_unfused(P, P, P, P, lens8, 2, 16, 2, 64, 16, mgr, 0, None) == eet.EET_ERR_CAPACITY   # 2 KB of scores
    assert eet.eet_bufmgr_query(mgr).buffers == 0                       # nothing was created on the way out
    assert L.eet_bufmgr_destroy(mgr) == eet.EET_OK


def test_stack_sizes_and_validation(eet):
    L = eet.lib()
    cfg = eet.make_config(1024, 16, 4096, 8, 512, 1024)
    # Section 3.1: 2*b*h*s*l elements, fp16
    assert eet.eet_stack_kv_cache_bytes(cfg, 24) == 2 * orc.kv_cache_elements(8, 1024, 1024, 24)
    ws1, wsn = eet.eet_workspace_bytes(cfg), eet.eet_stack_workspace_bytes(cfg, 24)
    # the layers share the scratch; the stack adds the two activation caches of 2*b*h*p elements (Section 3.1)
    assert wsn - ws1 == 2 * orc.activation_cache_elements(8, 1024, 512)
    assert eet.eet_stack_workspace_bytes(cfg, 0) == 0 and eet.eet_stack_kv_cache_bytes(cfg, 0) == 0
    ws = (eet.LayerWeights * 2)(eet.LayerWeights(*[0x10000] * 12), eet.LayerWeights(*[0x10000] * 12))
    h = C.c_void_p()
    assert L.eet_stack_create(C.byref(cfg), 0, ws, 0x100000, 1, C.byref(h)) == eet.EET_ERR_INVALID_ARG
    assert L.eet_stack_create(C.byref(cfg), 2, ws, 0x100000, 1, C.byref(h)) == eet.EET_OK and h.value
    P = 0x200000
    lens = (C.c_int32 * 2)(5, 600)
    assert L.eet_stack_decode_step(h, P, P, P, None) == eet.EET_ERR_STATE
    assert L.eet_stack_prefill(h, lens, 2, 512, P, P, P, None) == eet.EET_ERR_INVALID_ARG     # 600 > 512
    assert L.eet_stack_prefill(h, lens, 9, 512, P, P, P, None) == eet.EET_ERR_CAPACITY
    assert L.eet_stack_cache_lens(h, lens, None) == eet.EET_ERR_STATE
    assert L.eet_stack_encode(h, lens, 2, 512, P, P, P, None) == eet.EET_ERR_INVALID_ARG      # 600 > 512
    assert L.eet_stack_encode(h, lens, 2, 1024, P, P, P, None) == eet.EET_ERR_CAPACITY        # padded_len > max_prompt
    assert L.eet_stack_destroy(h) == eet.EET_OK
    bad = (eet.LayerWeights * 2)(eet.LayerWeights(*[0x10000] * 12), eet.LayerWeights(*[0x10000] * 11, 0))
    assert L.eet_stack_create(C.byref(cfg), 2, bad, 0x100000, 1, C.byref(h)) == eet.EET_ERR_INVALID_ARG and not h.value


def test_model_and_its_operators_validate(eet):
    L = eet.lib()
    cfg = eet.make_config(1024, 16, 4096, 8, 512, 1024)
    P = 0x200000
    # sizes: a zero bias of vocab_padded halfs, the per-sequence row indices and three [max_batch, hidden] rows -- no
    # prompt-sized buffer (Section 3.1: the embedding and the final output live in the stack's activation caches)
    mc = eet.ModelConfig(50257, 50304, 1024)
    ws = eet.eet_model_workspace_bytes(cfg, mc)
    assert 2 * 50304 + 3 * 2 * 8 * 1024 <= ws <= 2 * 50304 + 3 * 2 * 8 * 1024 + 4096
    assert eet.eet_model_workspace_bytes(cfg, eet.ModelConfig(50257, 50257, 1024)) == 0      # not a multiple of 64
    assert eet.eet_model_workspace_bytes(cfg, eet.ModelConfig(50257, 50240, 1024)) == 0      # padded < vocab
    lw = (eet.LayerWeights * 1)(eet.LayerWeights(*[0x10000] * 12))
    st = C.c_void_p()
    assert L.eet_stack_create(C.byref(cfg), 1, lw, 0x100000, 1, C.byref(st)) == eet.EET_OK
    mw = eet.ModelWeights(P, P, P, P)
    h = C.c_void_p()
    create = lambda s, c, m, w, wsp: L.eet_model_create(s, C.byref(c), C.byref(m), C.byref(w), wsp, C.byref(h))
    assert create(None, cfg, mc, mw, P) == eet.EET_ERR_INVALID_ARG
    assert create(st, eet.make_config(1024, 16, 4096, 8, 512, 2048), mc, mw, P) == eet.EET_ERR_INVALID_ARG   # another configuration
    assert create(st, cfg, eet.ModelConfig(50257, 50257, 1024), mw, P) == eet.EET_ERR_UNSUPPORTED_SHAPE
    assert create(st, cfg, eet.ModelConfig(0, 64, 1024), mw, P) == eet.EET_ERR_INVALID_ARG
    assert create(st, cfg, eet.ModelConfig(50257, 50304, 1000), mw, P) == eet.EET_ERR_INVALID_ARG          # max_pos < max_seq
    assert create(st, cfg, mc, eet.ModelWeights(P, P, 0, P), P) == eet.EET_ERR_INVALID_ARG
    assert create(st, cfg, mc, eet.ModelWeights(P + 2, P, P, P), P) == eet.EET_ERR_INVALID_ARG
    assert create(st, cfg, mc, mw, P + 16) == eet.EET_ERR_INVALID_ARG and not h.value                      # workspace alignment
    assert L.eet_model_prefill(None, None, 1, 1, P, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_model_decode_step(None, P, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_model_hidden_states(None, None, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_model_destroy(None) == eet.EET_OK
    assert L.eet_stack_destroy(st) == eet.EET_OK
    lens = (C.c_int32 * 2)(3, 9)
    assert L.eet_op_embedding(P, lens, 2, 8, 64, 100, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG        # len 9 > S 8
    assert L.eet_op_embedding(P, lens, 2, 16, 60, 100, 16, P, P, P, None) == eet.EET_ERR_UNSUPPORTED_SHAPE # hidden % 8
    assert L.eet_op_embedding(P, lens, 2, 16, 64, 100, 16, P, P + 4, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_embedding(None, lens, 2, 16, 64, 100, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_embedding_left_padded(P, lens, 2, 8, 64, 100, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG   # len 9 > S 8
    assert L.eet_model_prefill_left_padded(None, None, 1, 1, P, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_stack_prefill_left_padded(None, lens, 2, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_stack_encode(None, lens, 2, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_embedding_decode(P, None, 2, 64, 100, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_embedding_decode(P, P, 2, 64, 0, 16, P, P, P, None) == eet.EET_ERR_INVALID_ARG
    assert L.eet_op_argmax(P, 2, 100, 96, P, None) == eet.EET_ERR_INVALID_ARG                              # stride < vocab
    assert L.eet_op_argmax(P, 2, 100, 100, P, None) == eet.EET_ERR_INVALID_ARG                             # stride % 8
    assert L.eet_op_argmax(P, 2, 100, 104, None, None) == eet.EET_ERR_INVALID_ARG


def test_header_compiles_as_plain_c_and_links(eet, tmp_path):
    """include/eet.h is a C header: a C99 translation unit that includes it compiles without a warning under
    -Wall -Werror -pedantic, links against the library and gets the K/V cache size of Section 3.1 from it."""
    import shutil
    import subprocess
    gcc = shutil.which("gcc")
    if gcc is None:
        pytest.skip("no gcc")
    src = tmp_path / "use_header.c"
    src.write_text(
        '#include "eet.h"\n'
        '#include <stdio.h>\n'
        'int main(void) {\n'
        '    eet_layer_config c = {1024, 16, 4096, 8, 512, 1024, 1e-5f};\n'
        '    eet_bufmgr_t *m = 0;\n'
        '    (void)m;\n'
        '    printf("%lu %s\\n", (unsigned long)eet_kv_cache_bytes(&c), eet_last_error());\n'
        '    return eet_layer_destroy(0);\n'
        '}\n')
    exe = tmp_path / "use_header"
    libdir = os.path.dirname(eet.LIB_PATH)
    subprocess.run([gcc, "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-I", os.path.dirname(HEADER), str(src),
                    "-o", str(exe), "-L", libdir, "-l:libeet.so", f"-Wl,-rpath,{libdir}"], check=True)
    out = subprocess.run([str(exe)], check=True, capture_output=True, text=True).stdout.split()
    assert int(out[0]) == 2 * orc.kv_cache_elements(8, 1024, 1024, 1)
