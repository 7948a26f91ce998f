"""CPU oracle for the Harris coarsity pipeline: test infrastructure only.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import this
package; the GPU library and its Python binding never do.
"""
