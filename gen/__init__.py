"""Seeded synthetic inputs shared by the oracle's tests and the HIP path's tests/bench."""
from .cases import (C1, C2, C3, C4, C5, C4_PEAKY, EXTRA_WORKLOADS, WORKLOADS, Case, CaseSpec, make_case, tiny_spec,
                    mix64, normal12, stream_key, f32_to_bf16_bits, bf16_bits_to_f32,
                    f32_to_e4m3_bits, e4m3_bits_to_f32)
