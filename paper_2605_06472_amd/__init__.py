"""MI355X-native prefix-reuse prefill (attention over paged prefix KV + paged append +
host->pool page swap-in): HIP kernels behind a C-ABI library, with a thin Python binding.

``workloads`` draws the synthetic batches; ``binding`` loads ``libpbkv.so`` and marshals
arguments.  Nothing here computes attention on the CPU: without the built library or
without a GPU the calls raise.
"""
