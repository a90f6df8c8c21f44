"""CPU oracle (test infrastructure only).

Only the tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do.
"""
from .oracle import (DEAD, F32, BF16, build, build_detok_fst, fst_transduce, compile_compose,
                     compile_walk, mask_step, sample_step, sample_noise, gumbel_of_words, philox4x32_10, ln32, uniform, gumbel, advance_tokens, apply_terminals, minimize, compact, expand, concat_tables, max_threads,
                     PDA_STR, TokenEdges, pda_check_deterministic, pda_compile, pda_accepting, pda_step, pda_sample_step)

__all__ = ["DEAD", "F32", "BF16", "build", "build_detok_fst", "fst_transduce", "compile_compose",
           "compile_walk", "mask_step", "sample_step", "sample_noise", "gumbel_of_words", "philox4x32_10", "ln32", "uniform", "gumbel", "advance_tokens", "apply_terminals", "minimize", "compact", "expand", "concat_tables", "max_threads",
           "PDA_STR", "TokenEdges", "pda_check_deterministic", "pda_compile", "pda_accepting", "pda_step", "pda_sample_step"]
