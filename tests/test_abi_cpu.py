"""CPU-only checks of the boundary: the library loads and exports what the header declares."""
import ctypes
import os
import re

import pytest

import paper_2604_20470_amd as dr

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared(header="dynamicrad.h"):
    text = open(os.path.join(ROOT, "include", header)).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(dr_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_stage_calls():
    names = _declared()
    for n in ("dr_block_scores", "dr_build_mask", "dr_sparse_attn_fwd", "dr_create", "dr_destroy", "dr_last_error"):
        assert n in names


def test_library_exports_every_declared_symbol():
    lib = dr.load_library()
    for header in sorted(os.listdir(os.path.join(ROOT, "include"))):
        names = _declared(header)
        assert names, header
        for n in names:
            assert hasattr(lib, n), (header, n)
    assert dr.version().startswith("dynamicrad-gfx950")


def test_measurement_aids_are_not_in_the_product_header():
    product, probes = _declared(), _declared("dynamicrad_probe.h")
    assert probes == ["dr_clock_probe", "dr_mfma_mix_probe", "dr_mfma_probe"]
    assert not set(product) & set(probes)
    assert "dr_proxy_loss" in product


def test_struct_layouts_match_header():
    # dr_shape: 10 int32 + 3 int64 = 64 bytes; dr_mask_params: 4 doubles + 8 int32 = 64 bytes
    assert ctypes.sizeof(dr.Shape) == 64
    assert ctypes.sizeof(dr.MaskParams) == 64
    p = dr.MaskParams()
    assert (p.gamma, p.theta_c, p.theta_m, p.ratio_far, p.head_fuse) == (1.0, 0.15, 0.60, -1.0, 2)


def test_no_gpu_means_loud_failure_not_fallback():
    import torch
    if torch.cuda.is_available():
        pytest.skip("GPU present")
    with pytest.raises(dr.DRError):
        dr.Context(0)


def test_product_does_not_import_oracle():
    pkg = os.path.join(ROOT, "paper_2604_20470_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".hip", ".h", ".cpp")):
                src = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in src.replace("no CPU fallback", ""), f


def test_hand_scheduled_attention_kernel_compiles_without_spills_or_accumulator_copies():
    """k_attn_mfma_pair issues its matrix instructions through inline assembly, so the compiler neither knows their
    latency nor may move an accumulator while one of them still writes it.  A register allocation that spills, or that
    copies accumulation registers inside the chunk loop, computes garbage without any error: check the compiler's own
    report and the loop's code (cross-compiled here, nothing runs)."""
    import shutil
    import subprocess
    import tempfile
    from paper_2604_20470_amd import build as b
    if not (os.path.exists(b.HIPCC) or shutil.which(b.HIPCC)):
        pytest.skip("no hipcc")
    src = os.path.join(b.CSRC, "k_attn_mfma_pair.hip")
    with tempfile.TemporaryDirectory() as tmp:
        asm = os.path.join(tmp, "pair.s")
        r = subprocess.run([b.HIPCC, *[f for f in b.FLAGS if f != "-fPIC"], "-Rpass-analysis=kernel-resource-usage", "-S",
                            "--cuda-device-only", src, "-o", asm], capture_output=True, text=True)
        assert r.returncode == 0, r.stderr[-2000:]
        reports = [blk for blk in r.stderr.split("Function Name:")[1:]
                   if any(k in blk.splitlines()[0] for k in ("k_attn_mfma_pairE", "k_attn_mfma_quadE", "k_attn_mfma_octE"))]
        assert len(reports) == 3                      # block sizes 128, 64 and 32
        for report in reports:
            field = lambda name: int(re.search(name + r": (\d+)", report).group(1))
            assert field("VGPRs Spill") == 0 and field("SGPRs Spill") == 0
            assert field("VGPRs") <= 256 and field("AGPRs") <= 256
        lines = open(asm).read().splitlines()
    begins = [i for i, l in enumerate(lines) if "; chunk loop begin" in l]
    ends = [i for i, l in enumerate(lines) if "; chunk loop end" in l]
    assert len(begins) == 3 and len(ends) == 3
    for lo, hi in zip(begins, ends):
        loop = lines[lo:hi]
        assert 144 <= sum("v_mfma_f32_" in l for l in loop) <= 160    # two chunks of 72 slots (+ what drifts in from the drain)
        assert sum("v_mfma_f32_16x16x32_bf16" in l for l in loop) == 16   # the normaliser's eight per chunk, half length
        assert not any("v_accvgpr" in l for l in loop)
        assert not any("scratch_" in l or "buffer_store" in l for l in loop)
