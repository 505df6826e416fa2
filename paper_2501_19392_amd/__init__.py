"""AQUA-KV per-layer KV-cache encode / decode for MI355X (gfx950).

`paper_2501_19392_amd.binding` wraps the C-ABI library (libaquakv.so, built from
csrc/); `paper_2501_19392_amd.synth` produces seeded synthetic inputs.  Nothing
here computes the method on the CPU: without the built HIP library the binding
raises on import.
"""
__all__ = ["binding", "synth"]
