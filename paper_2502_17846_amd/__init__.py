"""MI355X-native GREM: streaming greedy min-edge-cut partitioning with refinement (Armada paper,
Sec. 4).  The computation lives in ``csrc/`` behind a C-ABI library; ``binding`` marshals
arguments to it, ``synth`` builds seeded inputs.  Importing the package loads no native code;
the first call into ``binding`` does, and fails loudly if the library is missing."""

__all__ = ["binding", "synth"]
