"""CPU-side checks of the C boundary: the library loads, exports what include/sop.h declares,
rejects work when no GPU is present, and its host atom builders agree with the oracle's."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import paper_2605_14929_amd as sop
from oracle import atoms as OA
import sop_inputs as si

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "sop.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(sop_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    names = _declared()
    assert {"sop_create", "sop_destroy", "sop_set_alphabet", "sop_set_pairs", "sop_workspace_bytes",
            "sop_pair_search", "sop_last_error"} <= set(names)
    L = sop.lib()
    for n in names:
        assert hasattr(L, n), n


def test_create_without_gpu_fails_loudly():
    import torch
    if torch.cuda.is_available():
        pytest.skip("a GPU is present")
    with pytest.raises(sop.SopError) as e:
        sop.Context(0)
    assert e.value.status == 6 and "no CPU fallback" in str(e.value)


def test_host_atom_builders_match_oracle_builders():
    for n in (3, 4, 5, 6):
        assert np.array_equal(sop.sop_atom_nf(n), OA.to_f32(OA.nf(n)))
        assert np.array_equal(sop.sop_atom_sh(n), OA.to_f32(OA.sh(n)))
    L = sop.sop_atom_sh(4)
    assert np.array_equal(sop.sop_atom_negate(L), OA.to_f32(OA.negate(L)))
    draws = si.normal_draws(1 << 16, 9)
    assert np.allclose(sop.sop_atom_bof(4, draws, 16, 20), OA.to_f32(OA.bof(4, draws, 16, 20)), rtol=0, atol=1e-6)
    x = OA.block_normalise(draws, 16)
    w = np.abs(si.normal_draws(x.size, 10)) + 0.1
    a = sop.sop_lloyd_1d(x, w, OA.nf(4), 7)
    b = OA.lloyd_1d(x, w, OA.nf(4), 7)
    assert np.allclose(a, b, rtol=0, atol=1e-9)


def test_builder_argument_errors():
    out = (C.c_float * 16)()
    assert sop.lib().sop_atom_nf(9, out) == 1
    assert sop.lib().sop_atom_nf(4, None) == 1
    assert sop.lib().sop_atom_sh(4, -1.0, 0.0, out) == 1


def test_search_table_matches_direct_search():
    # host logic of the library: the binned search table must reproduce the midpoint count for
    # every float near every code boundary, for each alphabet the GPU tests use
    draws = si.normal_draws(1 << 16, 4242)
    sets = [
        ["NF4", "SH4", "BOF4", "-NF4", "-SH4", "-BOF4"],
        ["NF5", "SH5", "BOF5", "-NF5", "-SH5", "-BOF5"],
        ["NF4", "SH5", "BOF4", "-NF5"],
        ["NF3", "SH6", "NF6"],
    ]
    for names in sets:
        nb, nc = sop.sop_check_alphabet(sop.build_alphabet(names, bof_draws=draws))
        assert 16 <= nb <= 512 and nc > 100000
    nb, _ = sop.sop_check_alphabet(sop.build_alphabet(["NF4", "SH4", "-NF4", "-SH4"]))
    assert nb <= 64                                                   # conflict-free table for the 4-bit atoms
    e2m3 = OA.to_f32(OA.exmy_grid(2, 3))
    three = np.array([-1.0, 0.0, 0.5], dtype=np.float32)
    odd = np.array([-3.0, -2.9, -0.1, 0.0, 0.7, 5.0], dtype=np.float32)
    sop.sop_check_alphabet([e2m3, sop.sop_atom_nf(4), three, sop.sop_atom_negate(three), odd])
    with pytest.raises(sop.SopError) as e:                            # boundaries closer than the finest table
        sop.sop_check_alphabet([np.array([-1.0, 0.0, 1e-4, 2e-4, 1.0], dtype=np.float32)])
    assert e.value.status == 3


def test_halved_table_values_and_entry_magnitudes():
    # The table holds half of every entry and the search kernels form a code boundary as the sum of two halves.
    # Host logic: (1) entries whose half is not exact are refused; (2) codebooks with entries of very different
    # magnitudes (where a binary64 mean could be rounded twice) and entries around binade boundaries still pass the
    # table self-check, which replays the summed-halves boundary against the midpoint count.
    with pytest.raises(sop.SopError) as e:
        sop.sop_check_alphabet([np.array([-1.0, 1e-44, 1.0], dtype=np.float32)])      # a subnormal entry: its half is not exact
    assert e.value.status == 3
    sop.sop_check_alphabet([np.array([-1.0, 0.0, 1.0], dtype=np.float32)])
    rng = np.random.default_rng(77)
    for _ in range(20):
        n = int(rng.integers(3, 17))
        mags = np.sort(np.exp(rng.uniform(np.log(1e-3), 0.0, size=n)).astype(np.float32))
        L = np.unique(np.concatenate([-mags[: n // 2 + 1][::-1], mags[n // 2:]])).astype(np.float32)
        try:
            sop.sop_check_alphabet([L])
        except sop.SopError as err:                                                   # only the spacing rule may refuse these
            assert "closely" in str(err)
    # neighbours more than 2^29 apart in magnitude, and entries exactly on powers of two
    sop.sop_check_alphabet([np.array([-1.0, -2.0 ** -31, 2.0 ** -3, 0.5], dtype=np.float32),
                            np.array([-1.0, -0.5, np.float32(0.5) + np.float32(2.0 ** -24), 1.0], dtype=np.float32)])


def test_binding_structures_match_the_header(tmp_path):
    """The ctypes mirrors of the header's structures have the header's sizes and field offsets (a C program that
    includes include/sop.h prints them)."""
    import subprocess
    from paper_2605_14929_amd import binding as B
    fields = {
        "sop_scale_fmt": (B.ScaleFmt, ["sign_bits", "exp_bits", "man_bits", "container_bits", "bias", "max_code"]),
        "sop_atom": (B._Atom, ["n_entries", "values"]),
        "sop_outputs": (B._Outputs, ["acos_pair", "acos_atom", "sel_words", "scale_code", "codes", "blk_cos", "blk_err", "blk_rank"]),
        "sop_layer": (B._Layer, None),
        "sop_weight_fmt": (B.WeightFmt, ["exp_bits", "man_bits", "bias", "max_code"]),
        "sop_layer_opts": (B._LayerOpts, ["n_p", "p_percent", "fit_entries", "fit_iters", "fit_bins", "fit_init", "weighted_fit", "fit_grid", "n_fit_grid", "pack"]),
        "sop_layer_result": (B._LayerResult, ["kind", "a", "b", "j", "p_percent", "acos", "n_entries_b", "table_b", "acos_fixed", "acos_atom", "acos_fitted", "n_bits"]),
    }
    lines = ['#include <stdio.h>', '#include <stddef.h>', '#include "sop.h"', 'int main(void) {']
    for name, (_, fl) in fields.items():
        lines.append(f'printf("{name} %zu\\n", sizeof({name}));')
        for f in fl or []:
            lines.append(f'printf("{name}.{f} %zu\\n", offsetof({name}, {f}));')
    lines += ['printf("SOP_MAX_ATOMS %d\\nSOP_MAX_ENTRIES %d\\nSOP_LAYER_MAX_P %d\\nSOP_LAYER_MAX_ATOMS %d\\nSOP_LAYER_MAX_PAIRS %d\\n", '
              'SOP_MAX_ATOMS, SOP_MAX_ENTRIES, SOP_LAYER_MAX_P, SOP_LAYER_MAX_ATOMS, SOP_LAYER_MAX_PAIRS);', 'return 0; }']
    src = tmp_path / "sizes.c"
    src.write_text("\n".join(lines))
    exe = tmp_path / "sizes"
    subprocess.check_call(["gcc", "-I", os.path.join(ROOT, "include"), "-o", str(exe), str(src)])
    got = dict(l.split() for l in subprocess.check_output([str(exe)], text=True).splitlines())
    for name, (cls, fl) in fields.items():
        assert int(got[name]) == C.sizeof(cls), name
        for f in fl or []:
            assert int(got[f"{name}.{f}"]) == getattr(cls, f).offset, (name, f)
    assert (int(got["SOP_MAX_ATOMS"]), int(got["SOP_MAX_ENTRIES"]), int(got["SOP_LAYER_MAX_P"])) == (B.MAX_ATOMS, B.MAX_ENTRIES, B.LAYER_MAX_P)
    assert (int(got["SOP_LAYER_MAX_ATOMS"]), int(got["SOP_LAYER_MAX_PAIRS"])) == (B.LAYER_MAX_ATOMS, B.LAYER_MAX_PAIRS)
