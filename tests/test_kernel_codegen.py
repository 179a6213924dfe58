"""CPU-only checks of what hipcc generated for gfx950 (cross-compiled here, no GPU needed): the properties the
performance of the streaming kernels rests on, which the optimiser has been seen to drop silently."""
import os
import re
import subprocess
import tempfile

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def asm():
    from paper_2006_07405_amd import build as B
    flags = [f for f in B.FLAGS if f not in ("-shared", "-fPIC")]
    text = ""
    with tempfile.TemporaryDirectory() as d:
        for k, src in enumerate(x for x in B.SOURCES if x.endswith(".hip")):
            out = os.path.join(d, f"k{k}.s")
            subprocess.check_call(["/opt/rocm/bin/hipcc"] + flags + ["--cuda-device-only", "-S", "-o", out, src],
                                  stderr=subprocess.DEVNULL)
            text += open(out).read()
    kernels = {}
    # a kernel's code: from its label to the end-of-function label (an early exit has an s_endpgm of its own)
    for m in re.finditer(r"^(_ZN5a2sgd\w+):.*?^\.Lfunc_end\d+:", text, flags=re.S | re.M):
        kernels[m.group(1)] = m.group(0)
    assert any("k_seg_apply" in k for k in kernels) and any("k_apply" in k for k in kernels)
    return text, kernels


def test_no_scratch_and_no_packed_fp32(asm):
    text, kernels = asm
    sizes = re.findall(r"\.private_segment_fixed_size:\s*(\d+)", text)
    assert sizes and all(s == "0" for s in sizes), "a kernel spills to scratch memory"
    assert not re.search(r"v_pk_(add|mul|fma)_f32", text)


def test_streaming_apply_stores_are_all_write_through_non_temporal(asm):
    _, kernels = asm
    # k_apply<MODE, HAS_E, NT, ...>: Lb1 in third place marks the streaming instantiations
    streaming = {k: v for k, v in kernels.items() if re.match(r"_ZN5a2sgd7k_applyILi[01]ELb[01]ELb1E", k)}
    assert len(streaming) >= 16
    for name, body in streaming.items():
        stores = re.findall(r"global_store_dwordx4[^\n]*", body)
        assert stores, name
        bad = [s for s in stores if not s.rstrip().endswith(" sc1 nt")]
        assert not bad, f"{name}: {len(bad)} of {len(stores)} 128-bit stores are not write-through non-temporal"
        # every hand-written store is followed by its two wait states (store-data hazard)
        lines = [l.strip() for l in body.splitlines() if l.strip() and not l.strip().startswith(";")]
        for k, l in enumerate(lines):
            if l.startswith("global_store_dwordx4") and l.endswith(" sc1 nt"):
                assert lines[k + 1].startswith("s_nop 1"), f"{name}: store without its wait states"


def test_every_hand_written_store_has_its_wait_states(asm):
    """All kernels of both files: the 128-bit store spelled in assembly must be followed by its two wait states, and
    the streaming instantiations of every pass that stores (NT = true: Lb1 among the template arguments) use it."""
    _, kernels = asm
    seen = 0
    for name, body in kernels.items():
        lines = [l.strip() for l in body.splitlines() if l.strip() and not l.strip().startswith(";")]
        for k, l in enumerate(lines):
            if l.startswith("global_store_dwordx4") and l.endswith(" sc1 nt"):
                seen += 1
                assert lines[k + 1].startswith("s_nop 1"), f"{name}: store without its wait states"
    assert seen > 100
    for pat in (r"_ZN5a2sgd15k_lazy_partialsILb1E", r"_ZN5a2sgd18k_lazy_materializeILb1E", r"_ZN5a2sgd13k_apply_signsILb1E",
                r"_ZN5a2sgd13k_error_signsILb1E", r"_ZN5a2sgd12k_dense_stepILb1E",
                r"_ZN5a2sgd11k_seg_applyILi[01]ELb[01]ELb1E", r"_ZN5a2sgd19k_seg_lazy_partialsILb1E",
                r"_ZN5a2sgd17k_seg_error_signsILb1E", r"_ZN5a2sgd17k_seg_apply_signsILb1E",
                r"_ZN5a2sgd17k_seg_materializeILb1E", r"_ZN5a2sgd27k_apply_replicas_per_workerILi[01]ELb[01]ELb1E",
                r"_ZN5a2sgd31k_seg_apply_replicas_per_workerILi[01]ELb[01]ELb1E"):
        names = [k for k in kernels if re.match(pat, k)]
        assert names, pat
        for name in names:
            stores = re.findall(r"global_store_dwordx4[^\n]*", kernels[name])
            assert stores and all(x.rstrip().endswith(" sc1 nt") for x in stores), name


def test_streaming_reduction_loads_are_non_temporal_and_batched(asm):
    _, kernels = asm
    name = next(k for k in kernels if re.match(r"_ZN5a2sgd16k_local_partialsILb1ELb1E", k))
    body = kernels[name]
    loads = re.findall(r"global_load_dwordx4[^\n]*", body)
    assert len(loads) >= 8 and all(l.rstrip().endswith(" nt") for l in loads)
    # in the main loop the eight loads of a tile are issued before the first wait on any of them
    loop = body[body.index("global_load_dwordx4"):]
    first_wait = loop.index("s_waitcnt vmcnt")
    assert loop[:first_wait].count("global_load_dwordx4") >= 8
