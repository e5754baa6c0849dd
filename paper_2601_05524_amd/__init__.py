"""MI355X-native verify / accept / retrieve / commit path of Double (arxiv 2601.05524).

`paper_2601_05524_amd.binding` wraps the C-ABI library (include/dbl.h);
`paper_2601_05524_amd.synth` holds the seeded synthetic-input generators.
"""
__all__ = ["binding", "synth"]
