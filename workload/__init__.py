"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

Holds no arithmetic of the method itself; see generate.py.
"""
from .generate import (LayerWeights, layer_weights, BLOCK, KIND_CHUNK, KIND_QUESTION, CONFIG_NAMES, RequestSpec, Spec, Workload,
                       bf16_bits, build, config, config_spec, custom, n_select_for, round_to_bf16,
                       SHIFT_SRC_TAB, SHIFT_DST_TAB, SHIFT_NTOK, SHIFT_DELTA,
                       SEG_REQ, SEG_KIND, SEG_START, SEG_NTOK, SEG_TAB, SEG_NSEL, SEG_TOK, SEG_SEL)
