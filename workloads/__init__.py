"""Seeded synthetic inputs for the encrypted-attention hot path.

This package only *draws* things: parameter presets (literal numbers), random
plaintext tensors shaped like GPT-2-small attention activations, the raw
randomness an encryptor consumes (ternary secret, rounded-Gaussian errors,
uniform ring elements) and uniformly random residue buffers that stand in for
ciphertexts and switching keys when only throughput is measured.  It contains
no ring arithmetic, no NTT, no modular multiplication: both the HIP library's
callers and the CPU oracle's callers may import it, and it imports neither.
"""
from .params import ParamSet, PRESETS, get_params
from .synth import (Stream, ternary_secret, gaussian_error, uniform_residues,
                    slot_values, attention_activations, pseudo_ciphertexts,
                    pseudo_switch_key, WORKLOADS, Workload)

from . import configs

__all__ = ["configs", "ParamSet", "PRESETS", "get_params", "Stream", "ternary_secret",
           "gaussian_error", "uniform_residues", "slot_values",
           "attention_activations", "pseudo_ciphertexts", "pseudo_switch_key",
           "WORKLOADS", "Workload"]
