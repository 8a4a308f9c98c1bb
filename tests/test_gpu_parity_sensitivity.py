"""How much the GPU parity checks see: the mistakes of test_pins_catch_mistakes.py are planted, one at a time, in a
copy of the ORACLE (never in the HIP path), and a battery of the small parity cases is run against the mistaken oracle
in this process.  The HIP path is right, so every planted mistake must make some comparison fail: a tolerance or a
case mix loose enough to let one through would show here.  With the unmodified oracle the battery passes."""
import ctypes
import importlib.util
import os
import sys
import time

import pytest

import oracle
from paper_2410_07590_amd import synth
from tests import test_gpu_parity as P
from tests import test_gpu_parity_softmax_range as S
from tests.test_pins_catch_mistakes import MISTAKES, PY_MISTAKES, SRC, _apply, _build, _package_copy

pytestmark = pytest.mark.gpu

PATCHED = ("online_prefill", "offline_chunk_prefill", "masked_prefill", "sequence_plan", "linear")


@pytest.fixture(scope="module")
def B():
    from paper_2410_07590_amd import binding
    binding.lib()
    return binding


def _battery(B):
    """Small cases of every entry point, cheapest first; raises on the first comparison that fails."""
    for mode in (synth.POS_REORDERED, synth.POS_COMPOSITE):
        P._ragged_case(B, 3, mode)                    # head_dim 64, group 8, a chunk used twice
        P._ragged_case(B, 0, mode)                    # ragged lengths, an empty chunk
        P.test_config1_fp32(B, mode)
    P._ragged_case(B, 2, synth.POS_REORDERED)         # one query head per KV head
    P._ragged_case(B, 0, synth.POS_REORDERED, layout=P.HALF)
    P.test_no_documents_and_noops(B)
    P.test_offline_ragged_chunks(B, "bf16")
    P.test_offline_ragged_chunks(B, "f32")
    for mode in (synth.POS_REORDERED, synth.POS_COMPOSITE):
        P.test_sequence_one_pass_ragged(B, mode)
    P.test_decode_batch_ragged(B, 0)
    P.test_linear_against_fp64_matmul(B, 3)
    P.test_linear_against_fp64_matmul(B, 9)
    S.test_first_visible_keys_in_one_half_of_a_key_step(B)      # logits that do not sit near zero
    S.test_logits_beyond_the_exponent_range(B)
    for seed in range(3):
        P.test_random_requests(B, seed)
        P.test_random_sequences(B, seed)


def _noticed(B):
    try:
        _battery(B)
    except Exception:   # an assertion of a comparison, or a shape the mistaken oracle cannot even produce
        return True
    return False


def test_battery_passes_with_the_oracle_as_it_is(B):
    _battery(B)


def test_mistakes_in_the_c_source_are_noticed(B, tmp_path, capsys):
    src = open(SRC).read()
    good = oracle.lib()
    missed = []
    try:
        for i, (name, old, new) in enumerate(MISTAKES):
            t0 = time.time()
            oracle._lib = ctypes.CDLL(_build(_apply(src, name, old, new), str(tmp_path / ("mistake%02d" % i))))
            hit = _noticed(B)
            with capsys.disabled():
                print("  planted: %-55s %s (%.1f s)" % (name, "noticed" if hit else "NOT NOTICED", time.time() - t0), flush=True)
            if not hit:
                missed.append(name)
    finally:
        oracle._lib = good
    assert not missed, "no GPU parity case notices: " + "; ".join(missed)


def test_mistakes_in_the_python_module_are_noticed(B, tmp_path, capsys):
    originals = {n: getattr(oracle, n) for n in PATCHED}
    missed = []
    try:
        for i, (name, old, new) in enumerate(PY_MISTAKES):
            d = _package_copy(tmp_path, "py%02d" % i, old, new)
            spec = importlib.util.spec_from_file_location("oracle_mistake%02d" % i, os.path.join(d, "oracle", "__init__.py"),
                                                          submodule_search_locations=[os.path.join(d, "oracle")])
            mod = importlib.util.module_from_spec(spec)
            sys.modules[spec.name] = mod
            spec.loader.exec_module(mod)
            t0 = time.time()
            for n in PATCHED:
                setattr(oracle, n, getattr(mod, n))
            hit = _noticed(B)
            with capsys.disabled():
                print("  planted: %-55s %s (%.1f s)" % (name, "noticed" if hit else "NOT NOTICED", time.time() - t0), flush=True)
            if not hit:
                missed.append(name)
    finally:
        for n, f in originals.items():
            setattr(oracle, n, f)
    assert not missed, "no GPU parity case notices: " + "; ".join(missed)
