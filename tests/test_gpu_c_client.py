"""The C ABI from a plain C11 program (no Python, no torch): one step, resampling and the reorder, checked in C."""
import os
import subprocess

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
CLIENT = os.path.join(ROOT, "tests", "c_client", "c_abi_client")


@pytest.mark.gpu
def test_c_client_runs_the_path():
    if not os.path.exists(CLIENT):                 # normally built by __graft_entry__.build(); a host-only gcc compile
        libdir = os.path.join(ROOT, "paper_2602_10273_amd")
        subprocess.run(["gcc", "-std=c11", "-O1", "-Wall", "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
                        "-I", os.path.join(ROOT, "include"), CLIENT + ".c", "-o", CLIENT, "-L", libdir, "-lpower_smc",
                        "-L/opt/rocm/lib", "-lamdhip64", "-Wl,-rpath," + libdir + ",-rpath,/opt/rocm/lib"], check=True)
    env = dict(os.environ)
    env["LD_LIBRARY_PATH"] = os.path.join(ROOT, "paper_2602_10273_amd") + ":/opt/rocm/lib:" + env.get("LD_LIBRARY_PATH", "")
    r = subprocess.run([CLIENT], capture_output=True, text=True, timeout=120, env=env)
    assert r.returncode == 0 and "c_abi_client ok" in r.stdout, r.stdout + r.stderr


def test_header_is_plain_c():
    """include/power_smc.h compiles as C11 on its own (no C++, no HIP or torch types in the signatures)."""
    src = '#include "power_smc.h"\nint main(void) { smc_config c; (void)c; return (int)sizeof(smc_status) == 0; }\n'
    r = subprocess.run(["gcc", "-std=c11", "-Wall", "-Werror", "-pedantic", "-fsyntax-only", "-I", os.path.join(ROOT, "include"),
                        "-x", "c", "-"], input=src, capture_output=True, text=True)
    assert r.returncode == 0, r.stderr
