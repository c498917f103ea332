"""CPU oracle for shifted sparse attention (S2-Attn). TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package; the product path (the HIP library and its Python binding) never does.
"""
