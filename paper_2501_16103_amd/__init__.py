"""MI355X-native statically batched MoE expert GEMM (hand-written HIP behind a C ABI).

`binding` forwards to libmoe_sb.so; `workloads` draws the seeded synthetic inputs;
`build` compiles the library.  Nothing here falls back to a CPU implementation.
"""
