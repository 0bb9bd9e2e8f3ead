"""ORACLE — test infrastructure only, never on the product path.

A plain, slow CPU interpreter of the tagged dataflow semantics of the paper, in float64,
written from the paper's definitions.  It shares no code with the HIP engine.  Only the
tests, the smoke check and the benchmark's CPU-baseline leg may import it.

Pins (see tests/test_oracle_*.py): the paper's factorial example and its transformed graph;
each semantic equation; Fibonacci closed forms and invocation counts; tree node counts;
the fire-exactly-once invariant; direct recursion; a left chain as an Elman RNN; finite
differences and closed-form gradients.  No part of the oracle is "parity unpinned".
"""
from .graph import Function, Program, transform, INT, FLOAT, VEC
from .interp import Interpreter, DEAD
from .autodiff import differentiate
from . import programs, ops, ops_bf16
