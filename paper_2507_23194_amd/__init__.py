"""MI355X-native output-equivalence check (the GEAK evaluator's tensor comparison, paper section 3.1).

`binding` wraps the C-ABI library built from `csrc/`; `synth` holds the seeded synthetic workloads.
Importing the package loads nothing; the library is loaded on the first call into `binding`
and that call raises if the HIP library has not been built.
"""
__all__ = ["binding", "synth"]
