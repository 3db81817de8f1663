"""MI355X-native evaluation of bit-accurate MMA arithmetic models (libmmaemu).

`paper_2511_10909_amd.binding` loads the HIP library and fails loudly if it is not built;
`paper_2511_10909_amd.synth` (numpy-only test inputs) and `.build` import without it.
"""
