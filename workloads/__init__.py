"""Seeded synthetic inputs (grammars, vocabularies, logits, token draws).

This package only *describes* inputs.  It contains no parsing, no automaton
construction and no masking arithmetic, so that both the CPU oracle and the
HIP library can consume the very same inputs without sharing any of the
method's code.
"""
from .rng import SplitMix64, stream, MASTER_SEED
from .grammar import Grammar, Lit, Rx
from . import grammars, vocab, configs
