"""MI355X-native hot path of monolithic forwarding with progressive cluster pruning:
`binding` wraps the HIP library (libprism.so), `workloads` draws the seeded synthetic inputs,
`build` compiles the library for gfx950."""
