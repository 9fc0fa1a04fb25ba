"""MI355X-native Compactor hot path (score -> select -> compact).

`paper_2507_08143_amd.compactor` is the binding of the HIP library (import it
explicitly: it fails loudly when libcompactor.so has not been built);
`paper_2507_08143_amd.workloads` draws the seeded synthetic inputs;
`paper_2507_08143_amd.build` compiles the library.
"""
