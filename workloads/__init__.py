"""Neutral workload descriptions shared by the tests, the benchmark, the oracle and the HIP path.

This package holds *data only*: operator programs written as plain lists of named ops, and seeded
generators for shapes and tensor values.  It contains none of the method's arithmetic (no operator
is evaluated here, no tile is planned, no byte of bytecode is produced), so that the CPU oracle and
the HIP virtual machine can both consume it without sharing any code with each other.
"""
from .programs import Program, Op, PROGRAMS, get_program  # noqa: F401
