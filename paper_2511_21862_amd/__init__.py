"""MI355X-native mixed-batch paged attention (offline decode + online prefill chunks over
one paged KV cache) and KV block copy: hand-written HIP kernels behind a C-ABI library.

`paper_2511_21862_amd.binding` is the thin ctypes binding over libooco.so; it raises at
load time when the HIP library has not been built.  `workloads` (seeded inputs) and
`accounting` (byte/flop bookkeeping) are importable without the library.
"""

__all__ = ["binding", "workloads", "accounting"]
