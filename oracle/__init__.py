"""CPU oracle for CSD verification.  Test infrastructure: imported by tests/, the smoke check and the
benchmark's CPU-baseline leg only; the GPU path never touches it."""
