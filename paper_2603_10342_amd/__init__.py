"""MI355X-native paged-KV attention for the three agent-serving request classes
(cold prefill, resume prefill, short GQA decode) behind a C-ABI library.

`paper_2603_10342_amd.binding` loads the HIP library and exposes its entry
points under the same names; `paper_2603_10342_amd.inputs` draws the seeded
synthetic workloads.  Importing the package itself loads nothing native.
"""

__all__ = ["binding", "inputs"]
