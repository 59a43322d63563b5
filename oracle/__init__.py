"""TEST INFRASTRUCTURE ONLY.  Plain, slow CPU oracle for one DFlash speculative-decoding step.
Nothing under the product package may import this; only tests/, the smoke check and the
bench's cpu_baseline leg do."""
