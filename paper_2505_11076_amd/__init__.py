"""MI355X-native Double Binary Factorization inference path (see the README).

The HIP library is loaded on first use of `paper_2505_11076_amd.binding`;
importing the package (for example to reach the seeded input generators in
`paper_2505_11076_amd.inputs`) touches no native code.
"""
__all__ = ["inputs", "binding"]
