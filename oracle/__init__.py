"""CPU oracle for the sparse-MoE feed-forward layer (test infrastructure only).

Only tests/, the smoke check and the bench's cpu_baseline leg import this
package; the GPU library and its Python binding never do.
"""
