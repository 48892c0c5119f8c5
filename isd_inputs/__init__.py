"""Seeded synthetic inputs for one introspective-strided-decoding (ISD) step.

This package only *draws inputs*: shapes, value distributions, block tables and
draft tokens of the five benchmark workloads.  It contains none of the method's
arithmetic (no attention, no acceptance rule, no sampler) and is the only code
shared by the CPU oracle's tests and the HIP path's tests / benchmark.
"""
from .configs import CONFIGS, ISDConfig, get_config, n_draft_for_stride
from .generate import (AcceptInputs, AttentionInputs, LoraInputs, make_accept_inputs,
                       make_attention_inputs, make_lora_inputs, bf16_bits, k_pages_in_operand_order, to_numpy)

__all__ = [
    "CONFIGS", "ISDConfig", "get_config", "n_draft_for_stride",
    "AcceptInputs", "AttentionInputs", "LoraInputs", "make_accept_inputs",
    "make_attention_inputs", "make_lora_inputs", "bf16_bits", "k_pages_in_operand_order", "to_numpy",
]
