"""The C-ABI library loads without a GPU, exports every symbol the header declares, and rejects
bad configurations before touching the device.  CPU only (no compute calls)."""
import ctypes as C
import os
import re

import pytest

from paper_2512_12928_amd import binding as B

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "ps.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(ps_[a-z_]+)\s*\(", text)))


def test_header_symbols_are_exported_and_bound():
    names = declared_symbols()
    assert "ps_step" in names and "ps_swap_out" in names and "ps_swap_in" in names
    L = B.lib()
    for n in names:
        assert hasattr(L, n), n
    assert sorted(B.EXPORTS) == names


def test_struct_sizes_match_header(tmp_path):
    """ctypes mirrors against sizeof() as a C compiler sees the header."""
    import subprocess
    src = tmp_path / "sz.c"
    src.write_text('#include <stdio.h>\n#include "ps.h"\nint main(void){printf("%zu %zu %zu %zu %zu\\n", sizeof(ps_layer_cfg), '
                   'sizeof(ps_batch), sizeof(ps_step_times), sizeof(ps_sched_cfg), sizeof(ps_batch_out));return 0;}\n')
    exe = tmp_path / "sz"
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Werror", "-I", os.path.join(ROOT, "include"), str(src), "-o", str(exe)])
    sizes = [int(x) for x in subprocess.check_output([str(exe)]).split()]
    assert sizes == [C.sizeof(B.ps_layer_cfg), C.sizeof(B.ps_batch), C.sizeof(B.ps_step_times),
                     C.sizeof(B.ps_sched_cfg), C.sizeof(B.ps_batch_out)]
    assert sizes[:3] == [84, 48, 36]


@pytest.mark.parametrize("kw", [dict(head_dim=64), dict(block_tokens=32), dict(n_q_heads=6, n_kv_heads=4),
                                dict(n_q_heads=34, n_kv_heads=2), dict(n_device_blocks=0), dict(out_dtype=7),
                                dict(decode_chunk=48), dict(decode_chunk=16), dict(softmax_scale=-1.0),
                                dict(decode_waves=-1), dict(swap_dma_runs=-1), dict(plan_decode_share=2.0)])
def test_create_rejects_bad_cfg_without_a_device(kw):
    args = dict(n_q_heads=8, n_kv_heads=2, n_device_blocks=64)
    args.update(kw)
    with pytest.raises(B.PsError) as e:
        B.ps_create(**args)
    assert e.value.code == B.PS_EINVAL and str(e.value)


def test_null_arguments_are_errors_not_crashes():
    L = B.lib()
    assert L.ps_create(None, None) == B.PS_EINVAL
    assert L.ps_step(None, None, None, None, None, None, None, None, 0, None, 0) == B.PS_EINVAL
    assert L.ps_step_next_layer(None, None, None, None, None, None, None, 0, None, 0) == B.PS_EINVAL
    n, t = C.c_int32(), C.c_uint64()
    assert L.ps_swap_out(None, None, None, 0, 0, None, None, None, C.byref(n), C.byref(t)) == B.PS_EINVAL
    assert L.ps_ticket_wait(None, 1) == B.PS_EINVAL
    L.ps_destroy(None)
