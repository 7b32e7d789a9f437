"""MI355X-native MLA decode attention (split-KV + LSE combine) behind a C ABI.

``from paper_2506_01969_amd import mla`` loads the HIP library lazily on first call.
"""
