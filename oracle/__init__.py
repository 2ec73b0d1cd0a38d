"""CPU oracle for the encrypted-attention hot path -- TEST INFRASTRUCTURE ONLY.

Only the test suite, the smoke check and the benchmark's cpu_baseline leg may
import this package.  It shares nothing with the HIP library.  Contents:

  bfv.Oracle        ctypes wrapper over src/bfv_oracle.c: the evaluator
                    operations (mul, keyswitch, relin, rotate, add, mul_plain)
                    written as their definitions over the integers.
  client.Client     host-side key generation, slot encoding, encryption and
                    decryption (the party that holds the secret key).
  attention         the cache append and the decode / prefill attention
                    products as plain sequences of evaluator operations.
  run_configs       the five benchmark configurations end to end (used to write the
                    digests under tests/golden/ and by the CPU baseline).
"""
from .bfv import Oracle, load_library
from .client import Client
from . import attention
from . import run_configs

__all__ = ["Oracle", "Client", "attention", "run_configs", "load_library"]
