"""CPU checker for the encoder task.  Test infrastructure: imported only by tests/, the
smoke check and the benchmark's CPU-baseline leg -- never by the GPU library's binding."""
