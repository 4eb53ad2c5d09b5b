"""CPU fp64 oracle of the MoE expert layer.  Test infrastructure: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg only; never by the product path."""
