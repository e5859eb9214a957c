"""The generated assembly loop: the committed attn_loop_gfx950.inc is what the generator writes now (a stale
file would build an older loop), and the generator's own checks (register budget, slot distances between an
MFMA and the first use of its result, vector work behind the last MFMA) hold for every configuration."""
import importlib.util
import os

HERE = os.path.dirname(os.path.abspath(__file__))
CSRC = os.path.join(HERE, "..", "paper_2502_18137_amd", "csrc")


def load_generator():
    spec = importlib.util.spec_from_file_location("gen_attn_loop", os.path.join(CSRC, "gen_attn_loop.py"))
    mod = importlib.util.module_from_spec(spec)
    spec.loader.exec_module(mod)
    return mod


def test_committed_loop_is_current():
    gen = load_generator()
    with open(os.path.join(CSRC, "attn_loop_gfx950.inc")) as f:
        committed = f.read()
    assert gen.generate() == committed


def test_register_budgets():
    gen = load_generator()
    for D in (64, 128):
        for dt, qk16 in (("f16", False), ("bf16", False), ("fp8", False), ("f16", True), ("bf16", True)):
            c = gen.Cfg(D, dt, qk16=qk16)
            assert c.NVGPR <= 256
            # pinned scalar registers stay below the ones the ABI reserves at the top (vcc, flat_scratch, xnack)
            assert max(c.sg.values()) < 96
            # every tuple the MFMAs use starts at an even register
            assert c.O % 2 == 0 and c.Q % 2 == 0 and c.RG % 2 == 0
