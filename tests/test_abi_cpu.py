"""No-GPU checks of the boundary: the shared library loads and exports every
entry point the header declares; the binding's name list matches the header."""
import ctypes
import os
import re

from paper_2509_09424_amd import binding

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "ensi.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ensi_[a-z0-9_]+)\s*\(", text)))


def test_header_and_binding_agree():
    assert _declared() == sorted(binding.EXPORTED)


def test_library_exports_every_declared_symbol():
    if not os.path.exists(binding.LIB_PATH):
        import __graft_entry__
        __graft_entry__.build()
    lib = ctypes.CDLL(binding.LIB_PATH)
    for name in _declared():
        assert hasattr(lib, name), name


def test_error_codes_and_null_handling_without_gpu():
    lib = binding.load()
    # argument validation happens before any device call
    assert lib.ensi_ctx_create(None, None) == -1
    assert lib.ensi_last_error(None) == b"null context"
    bad = binding._Params(3, 50, 2, 60, 1, 1, 40, 0)  # log_n below the supported range
    h = ctypes.c_void_p()
    assert lib.ensi_ctx_create(ctypes.byref(bad), ctypes.byref(h)) == -1 and not h.value


def test_null_arguments_of_the_later_entry_points_without_gpu():
    """Every entry point rejects null handles before it touches the device."""
    lib = binding.load()
    n = None
    d = ctypes.c_double
    assert lib.ensi_pt_set_scale(n, d(1.0)) == -1
    assert lib.ensi_ct_drop_limbs(n, 1) == -1
    assert lib.ensi_encode_at(n, n, 1, 1, 1, d(2.0), n) == -1
    assert lib.ensi_pmult_sum_rescale(n, n, n, n, n, n, 1, n, n) == -1
    assert lib.ensi_set_pmult_mode(n, 0) == -1
    assert lib.ensi_block_masks(n, 1, 1, 2, n) == -1
    assert lib.ensi_merge(n, n, n, 1, n, n) == -1
    assert lib.ensi_rope_plaintexts(n, n, n, 1, 2, n) == -1
    assert lib.ensi_rope(n, n, n, n, n, n) == -1
    assert lib.ensi_relin_keygen(n, n, n, ctypes.c_uint64(0), n) == -1
    assert lib.ensi_mult_sum_relin_rescale(n, n, n, n, n, n, n, 1, n, n) == -1
    assert lib.ensi_one_hot_masks(n, 1, 2, n) == -1
    assert lib.ensi_periodic_masks(n, 2, 1, 2, n) == -1
    assert lib.ensi_replicate(n, n, n, n, n, n, 1, n, n) == -1
    assert lib.ensi_ccmm(n, n, n, n, n, n, 2, n, n) == -1
    assert lib.ensi_block_start_mask(n, 2, 2, n) == -1
    assert lib.ensi_fill_steps(0, 8, 1, n, 0) == -1 and lib.ensi_fill_steps(1, 8, 0, n, 0) == -1
    assert lib.ensi_fill_steps(1, 32, -1, n, 0) == 7  # a pure host query: -1 -2 -3 | -4 -8 -12 | -16
    assert lib.ensi_ccmm_blocks(n, n, n, n, n, 2, n, 1, n, n, n) == -1
    assert lib.ensi_block_head_mask(n, 4, 2, 2, n) == -1
    assert lib.ensi_ccmm_bsgs(n, n, n, n, n, 4, 2, n, n, n, n, 1, n, n, n, n) == -1
    assert lib.ensi_segment_masks(n, 4, 2, 2, n) == -1
    assert lib.ensi_ccmm_segment(n, n, n, n, n, 4, 2, 2, 0, n, n, n, n) == -1
    assert lib.ensi_ccmm_left_giant_steps(n, n, n, 4, 2, 0, n, n) == -1
    assert lib.ensi_diagonalise_weights(n, n, n, 4, 2, 2, n, 0, n, n) == -1
    assert lib.ensi_ccmm_av(n, n, n, n, n, 4, 2, 2, 0, n, n, n) == -1


def test_null_arguments_of_key_exchange_and_prepared_weights_without_gpu():
    lib = binding.load()
    n = None
    d = ctypes.c_double
    assert lib.ensi_sk_import(n, n, n) == -1 and lib.ensi_sk_export(n, n, n) == -1
    assert lib.ensi_pk_import(n, n, n) == -1 and lib.ensi_pk_export(n, n, n) == -1
    assert lib.ensi_gk_import(n, n, 1, n) == -1 and lib.ensi_gk_export(n, n, 1, n) == -1
    assert lib.ensi_gk_elements(n, n, 0) == -1
    assert lib.ensi_ct_checksum(n, n, n, n) == -1
    assert lib.ensi_weights_prepare(n, n, 1, 1, 1, 0, 1, n) == -1
    assert lib.ensi_ternary_matmul_prepared(n, n, n, n, n, n) == -1
    assert lib.ensi_rescale_ternary_matmul_prepared(n, n, d(0.5), n, n, n) == -1
    assert lib.ensi_matrix_rate_probe(n, d(0.1), n, n) == -1
    lib.ensi_weights_free(n)  # a null handle is ignored
