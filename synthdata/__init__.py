"""Seeded synthetic inputs shared by the CPU oracle's tests and the GPU library's tests."""
from .gen import (BASE_CHUNK, BASE_SEED, CONFIGS, Config, Mixture, STREAM_BASE0, STREAM_INIT,
                  STREAM_QUERY, STREAM_TRAIN, base_chunk, draw_without_replacement, gauss_table,
                  gen_base, gen_vectors, make_mixture, mix64, stream_key, hash_at)
