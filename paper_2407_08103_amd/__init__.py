"""Token-level constraint automata for LM decoding (arXiv 2407.08103) on AMD CDNA4 / gfx950.

The package is a thin binding over the C-ABI library declared in include/tdfa.h.
"""
from .binding import (PATH_AUTO, PATH_PAIRS, PATH_STAGED, PATH_WALK, BF16, advance_tokens, DEAD, F32, NO_TOKEN, CharDFA, Table, TdfaError, Vocab, allow_row_words,
                      compile_stacked, compile_token_dfa, dfa_union, dfa_union_host, lib, mask_step, mask_step_noalloc, plan_describe, sample_noise, sample_step, table_apply_terminals, table_concat, table_minimize, table_pack, table_pack_arrays, table_wrap)
from .binding import CharPDA, TokenPDA, compile_token_pda, pda_step, pda_sample_step, PDA_STRING, trim
from .build import build

__all__ = ["PATH_AUTO", "PATH_PAIRS", "PATH_STAGED", "PATH_WALK", "BF16", "advance_tokens", "DEAD", "F32", "NO_TOKEN", "CharDFA", "Table", "TdfaError", "Vocab", "allow_row_words",
           "compile_stacked", "compile_token_dfa", "dfa_union", "dfa_union_host", "lib", "mask_step", "mask_step_noalloc", "plan_describe", "sample_noise", "sample_step", "table_apply_terminals", "table_concat", "table_minimize", "table_pack", "table_pack_arrays", "table_wrap", "build", "CharPDA", "TokenPDA", "compile_token_pda", "pda_step", "pda_sample_step", "PDA_STRING", "trim"]
