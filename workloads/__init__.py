"""Seeded synthetic inputs for the batched RNNLM step.

This module only draws random numbers and shuffles/gathers arrays: it holds none
of the method's arithmetic (no recurrent update, no projection, no log-sum-exp,
no grouping of equal keys).  Both the CPU oracle's tests and the GPU library's
tests/bench take their inputs from here, so the two sides see identical bits.

The five workloads stand in for the paper's corpora (WSJ eval92/dev93 and an
in-house set, Section 5.1), which are not available.  Their shapes follow the
paper's statistics: a few thousand new word hypotheses per frame (Section 3.2),
most lookups redundant (Section 5.2), vocabularies from 20 K up to very large.
No item of any corpus is reproduced.
"""
from .configs import (CONFIGS, Workload, make_model, make_step_inputs, bounded_zipf_ids,
                      round_to_bf16, bf16_bits, pack_history_id, DecodeTrace)

__all__ = ["CONFIGS", "Workload", "make_model", "make_step_inputs", "bounded_zipf_ids",
           "round_to_bf16", "bf16_bits", "pack_history_id", "DecodeTrace"]
