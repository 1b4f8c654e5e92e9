"""Writes tests/golden/operand_sigma.txt: the operand noise floor sigma of a small bf16 model.

sigma = rms, over the rows of the first forward of a block (all masked, behind a cached prompt), of the
difference in max logit between two evaluations of the oracle that differ only in cfg["operand_dtype"]:
None (nothing rounded) and torch.bfloat16 (every activation that enters a matrix product rounded to bf16
first).  The bf16 GPU tolerances are multiples of this quantity, so the places where the oracle rounds
set them: a rounding point that is dropped or added changes sigma, and tests/test_oracle_pins.py
compares a fresh evaluation with the value stored here.

Calls only oracle/ (and the seeded input generator).  Run: python tests/golden/make_operand_sigma.py
"""
import os
import sys

import torch

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)

from oracle import decode, model  # noqa: E402
from paper_2510_04147_amd import synth  # noqa: E402

SHAPE = dict(dtype="bf16", n_layers=2, d_model=256, n_q_heads=4, n_kv_heads=2, head_dim=64, d_ffn=768, vocab=1024)
WEIGHT_SEED, PROMPT_SEED, PROMPT_LEN, BLOCK, STD = 31, 32, 40, 32, 0.05


def max_logits(operand_dtype):
    cfg = dict(synth.model_config("tiny", **SHAPE), operand_dtype=operand_dtype)
    w = synth.gen_weights(cfg, WEIGHT_SEED, std=STD)
    prompt = synth.gen_prompt(cfg, PROMPT_SEED, PROMPT_LEN)
    cache = model.KVCache(cfg["n_layers"])
    _, kv = model.forward_segment(w, cfg, prompt, 0, cache, torch.float64, need_logits=False)
    cache.append(kv)
    logits, _ = model.forward_segment(w, cfg, [cfg["mask_id"]] * BLOCK, PROMPT_LEN, cache, torch.float64)
    return decode.predict(logits, cfg["mask_id"])[1]


def sigma():
    a, b = max_logits(None), max_logits(torch.bfloat16)
    return float(((a - b) ** 2).mean().sqrt())


if __name__ == "__main__":
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "operand_sigma.txt")
    with open(path, "w") as f:
        f.write("# Operand noise floor of the oracle (fp64) on the small bf16 model of make_operand_sigma.py:\n")
        f.write("# rms difference in max logit between operand_dtype None and bfloat16, first forward of a block.\n")
        f.write("# Written by tests/golden/make_operand_sigma.py, which calls only oracle/.\n")
        f.write(f"{sigma():.12e}\n")
    print(open(path).read())
