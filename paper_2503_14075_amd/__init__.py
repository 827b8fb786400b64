"""MI355X-native hot path of TwigVLM / TwigVLM++ decoding over a pruned
multimodal KV cache: twig-guided token pruning (score, top-R select, stable
compaction) and tree-based self-speculative verification (tree-masked
attention, greedy acceptance walk).

`paper_2503_14075_amd.binding` loads the HIP library and exposes one Python
function per C-ABI entry point; importing it raises if the library has not
been built.  `paper_2503_14075_amd.workloads` generates the seeded synthetic
inputs and needs neither the library nor a GPU.
"""
