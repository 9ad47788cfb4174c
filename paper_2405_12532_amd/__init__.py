"""MI355X-native prefill layer step of PyramidInfer (arXiv 2405.12532).

`paper_2405_12532_amd.binding` wraps the C-ABI library built from `csrc/`;
`paper_2405_12532_amd.synth` makes the seeded synthetic inputs.  Importing the
package loads nothing native; the binding raises if the library is missing.
"""
