"""MI355X-native deep Q-learning training step (arxiv 1804.05834).

`paper_1804_05834_amd.dqn` is the thin ctypes binding over the C-ABI library built from
`csrc/`; `paper_1804_05834_amd.synth` holds the seeded synthetic-input generators.  Nothing is
imported eagerly, so the generators can be used without the HIP library.
"""
__all__ = ["dqn", "synth"]
