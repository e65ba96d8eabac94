"""MI355X-native TIDE router hot path: fused RMSNorm + router evaluation + earliest-exit
selection (libtide_route), its Python binding, seeded synthetic workloads and exit
statistics.  ``tide_route`` needs torch and the built HIP library; ``synth`` and
``stats`` are numpy only."""
