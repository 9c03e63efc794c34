"""Shared helpers of the GPU parity tests: the same seeded inputs go to the oracle and the library."""
import numpy as np

from oracle import decoder
from paper_2510_19705_amd import inputs


def oracle_spec(shape):
    return decoder.Spec(shape["n_layers"], shape["d"], shape["n_q"], shape["n_kv"], shape["hd"], shape["ffn"],
                        shape["vocab"], inputs.ROPE_BASE, inputs.EPS)


def oracle_decoder(shape, weights, max_len):
    return decoder.Decoder(oracle_spec(shape), weights, max_len)


def gpu_model(shape, weights, bf16, max_seq, max_rows, rows_copy_layers=0):
    from paper_2510_19705_amd import hsd
    m = hsd.Model(shape, hsd.BF16 if bf16 else hsd.F32, max_seq, max_rows, inputs.ROPE_BASE, inputs.EPS, rows_copy_layers)
    m.load(weights)
    return m


def say(*a):
    print(*a, flush=True)
