"""Host-side checks of the C ABI that need no GPU: the library loads, exports every declared symbol,
sizes its workspace and rejects bad arguments before touching a device."""
import os
import re

import pytest

from paper_2602_10273_amd import binding as smc

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    text = open(os.path.join(ROOT, "include", "power_smc.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(smc_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = smc.lib()
    names = _declared()
    assert set(names) == set(smc.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_workspace_size_and_config_validation():
    ok = smc.make_config(16, 8, 152064, 512, "bf16", 0.5, 1, 56, 4, 2048, 128, 2)
    n = smc.smc_workspace_bytes(ok)
    assert n > 0 and n % 256 == 0 and n < 64 << 20
    bad = [dict(B=0), dict(N=0), dict(N=2000), dict(V=0), dict(T_max=6), dict(logits_dtype=5), dict(kappa=1.5),
           dict(kappa=-0.1), dict(kv_D=3), dict(kv_elem_bytes=3), dict(kv_tensors=100000)]
    for kw in bad:
        c = smc.make_config(16, 8, 152064, 512, "bf16", 0.5, 1, 56, 4, 2048, 128, 2)
        for k, v in kw.items():
            setattr(c, k, v)
        assert smc.smc_workspace_bytes(c) == 0, kw
        with pytest.raises(smc.SMCError):
            smc.smc_init(c, 256, 1 << 30)


def test_init_argument_errors_come_before_any_device_use():
    c = smc.make_config(1, 4, 8, 8, "f32", 0.5, 1)
    n = smc.smc_workspace_bytes(c)
    with pytest.raises(smc.SMCError) as e:
        smc.smc_init(c, None, n)
    assert e.value.status == 1            # SMC_E_NULL
    with pytest.raises(smc.SMCError) as e:
        smc.smc_init(c, 264, n)           # misaligned workspace
    assert e.value.status == 4
    with pytest.raises(smc.SMCError) as e:
        smc.smc_init(c, 256, n - 1)       # too small
    assert e.value.status == 2
    assert smc.smc_status_str(0) == "ok" and smc.smc_status_str(4) == "bad alignment"
    for fn, args in [(smc.lib().smc_step, (None, None, 8, 1, 1.0, 1.0, -1.0, None)),
                     (smc.lib().smc_ess, (None, None, None)), (smc.lib().smc_destroy, (None,)),
                     (smc.lib().smc_kv_reindex, (None, None, None, 0, 0))]:
        assert fn(*args) == 1             # null context
