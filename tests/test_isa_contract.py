"""Build-time check of an assumption the SpMV kernel makes about its own
generated code.

The kernel copies x into LDS with direct-to-LDS loads, then issues the weight
loads, then waits with ``s_waitcnt vmcnt(N)`` before a plain ``s_barrier``.
Loads complete in issue order, so the wait covers the copy of x exactly when at
least N vector-memory loads were issued after the last direct-to-LDS load.
The compiler does not track that dependency itself, so this test reads the
assembly the compiler emits for OUR sources (``hipcc -S``) and checks N against
the instruction stream of every instantiation.  No GPU needed.
"""
import os
import re
import subprocess
import tempfile
from concurrent.futures import ThreadPoolExecutor

import pytest

from paper_1811_00206_amd import build as bs_build

SOURCES = ["bs_spmv_f32.hip", "bs_spmv_f16.hip", "bs_spmm_f32.hip", "bs_spmm_f16.hip",
           "bs_spmm_rows.hip", "bs_spmv_slab.hip", "bs_spmv_wide.hip", "bs_spmm_wide.hip"]


def _assembly(src):
    out = tempfile.NamedTemporaryFile(suffix=".s", delete=False).name
    flags = [f for f in bs_build.FLAGS if f not in ("-fPIC",)]
    subprocess.check_call([bs_build.HIPCC, *flags, "-S", "--cuda-device-only", "-o", out,
                           os.path.join(bs_build.CSRC, src)],
                          stderr=subprocess.DEVNULL)
    text = open(out).read()
    os.unlink(out)
    return text


def _kernels(text):
    """name -> list of instruction lines (plus the "; bs_pin" markers that
    pin_order() leaves), for every spmv_kernel / spmm_kernel / spmm_rows_kernel
    instantiation."""
    out = {}
    cur = None
    for line in text.splitlines():
        m = re.match(r"^(_ZN2bs(?:11sp(?:mv|mm)_kernel|16spmm_rows_kernel)\w+):", line)
        if m:
            cur = m.group(1)
            out[cur] = []
            continue
        if cur is not None:
            s = line.strip()
            if s.startswith("s_endpgm"):
                cur = None
            elif s.startswith("; bs_pin"):
                out[cur].append("bs_pin")
            elif s and not s.startswith((";", ".")):
                out[cur].append(s)
    return out


def _is_vmem_load(ins):
    return ins.startswith(("global_load_", "buffer_load_", "flat_load_", "scratch_load_"))


@pytest.fixture(scope="module")
def texts():
    with ThreadPoolExecutor(4) as ex:
        return list(ex.map(_assembly, SOURCES))


@pytest.fixture(scope="module")
def kernels(texts):
    ks = {}
    for t in texts:
        ks.update(_kernels(t))
    return ks


def test_every_instantiation_is_present(kernels):
    # 3 chunk widths for fp32 + 4 for fp16, 7 group widths; 7 in-flight depths for
    # SpMV, plus 4 group widths and 2 depths of the fused LSTM step; 5 group widths
    # and 2 depths for SpMM
    # ... and for 16-bit offsets: 2 chunk widths per type, 4 group widths, 3 depths for SpMV;
    # 2 chunk widths, 5 group widths, 2 depths for SpMM
    assert sum("spmv_kernel" in n for n in kernels) == (3 + 4) * 7 * 7 + (3 + 4) * 4 * 2 + 2 * 2 * 4 * 3
    assert sum("spmm_kernel" in n for n in kernels) == (3 + 4) * 5 * 2 + 2 * 2 * 5 * 2
    # one lane per (row, column group): chunk widths only
    assert sum("spmm_rows_kernel" in n for n in kernels) == 3 + 4 + 2 * 2


def test_wait_before_barrier_covers_the_copy_of_x(kernels):
    for name, ins in kernels.items():
        barrier = next(i for i, s in enumerate(ins) if s.startswith("s_barrier"))
        dma = [i for i, s in enumerate(ins[:barrier]) if s.startswith("global_load_lds")]
        assert dma, f"{name}: no direct-to-LDS load before the barrier"
        pins = [i for i, s in enumerate(ins[:barrier]) if s == "bs_pin"]
        assert len(pins) >= 2, f"{name}: pin markers missing"
        first, second = pins[-2], pins[-1]
        # every copy of x is issued before the first pin, the weight loads sit between
        # the pins, and the wait follows the second pin
        assert dma[-1] < first, f"{name}: a direct-to-LDS load follows the first pin"
        waits = [i for i in range(second, barrier) if ins[i].startswith("s_waitcnt")
                 and "vmcnt" in ins[i]]
        assert waits, f"{name}: no vmcnt wait between the weight loads and the barrier"
        n_allowed = int(re.search(r"vmcnt\((\d+)\)", ins[waits[-1]]).group(1))
        issued = sum(_is_vmem_load(s) for s in ins[first:second])
        assert n_allowed <= issued, (
            f"{name}: waits for vmcnt({n_allowed}) but only {issued} loads sit between the "
            "pins: x may not have landed at the barrier")
        assert not any(_is_vmem_load(s) for s in ins[second:barrier]), (
            f"{name}: a load between the second pin and the barrier would break the count")
        # no LDS read before the barrier at all
        assert not any(s.startswith("ds_read") for s in ins[:barrier]), name


def test_no_kernel_spills_registers(texts):
    """Every SpMV / SpMM instantiation fits its register budget: a spill would put scratch
    memory traffic into the inner loops (seen once with 16 gathers in flight)."""
    n = 0
    for t in texts:
        for m in re.finditer(r"\.(vgpr|sgpr)_spill_count:\s+(\d+)", t):
            n += 1
            assert int(m.group(2)) == 0, f"{m.group(1)} spills: {m.group(2)}"
        for m in re.finditer(r"\.private_segment_fixed_size:\s+(\d+)", t):
            assert int(m.group(1)) == 0, "a kernel uses scratch memory"
    assert n > 0
