"""MI355X-native rectified block-sparse attention (hand-written HIP behind a C-ABI).

``paper_2511_19835_amd.binding`` marshals arguments to ``librsa.so``; ``synth`` draws the
seeded synthetic inputs. Nothing in this package computes the method on the CPU.
"""
__all__ = ["binding", "synth"]
