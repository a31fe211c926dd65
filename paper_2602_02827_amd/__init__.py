"""MI355X-native Col-Bandit scoring path: HIP kernels behind a C-ABI library.

`paper_2602_02827_amd.binding` is the thin ctypes layer over the C-ABI;
`paper_2602_02827_amd.synth` holds the seeded input generators.  Importing the
package does not load the HIP library; the binding loads it on first use and
raises if it has not been built.
"""
__all__ = ["binding", "synth"]
