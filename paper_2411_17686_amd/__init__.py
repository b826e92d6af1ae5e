"""MI355X-native FiCoCo (filter / correlate / compress) token-reduction step.

`paper_2411_17686_amd.ficoco` is the thin ctypes binding over the C-ABI library built from
`csrc/`; `paper_2411_17686_amd.synth` holds the seeded input generators.  Importing the
package loads nothing: the binding opens the shared library on first use and raises if it
has not been built.
"""
__all__ = ["ficoco", "synth"]
