"""MI355X-native rANS intermediate-feature codec (HIP kernels behind a C ABI).

``paper_2511_11664_amd.synth`` draws the synthetic workloads; ``paper_2511_11664_amd.binding``
loads ``librans_if.so`` (built from ``csrc/``) and marshals arguments.  Importing the package
does not load the library; the first call into ``binding`` does, and raises if it is missing.
"""
