"""MI355X-native paged KV-cache data path: paged decode attention and KV-block pack/restore."""

# The binding (kvflow) needs torch and the built library; the input generators (workloads) need
# neither.  Import them as submodules: paper_2601_22438_amd.kvflow, paper_2601_22438_amd.workloads.
