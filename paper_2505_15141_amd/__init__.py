"""MI355X-native hot path of BanditSpec (arXiv 2505.15141): one speculative-decoding round
(draft proposal, target verification forward, accept/reject sampling) plus the host-side
UCBSpec / EXP3Spec arm selection, as a C-ABI HIP library with a thin ctypes binding.

`from paper_2505_15141_amd import binding` loads the built library (and fails loudly if it is missing).
`paper_2505_15141_amd.synth` holds the seeded input generators only.
"""
