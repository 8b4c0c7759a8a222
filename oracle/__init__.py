"""CPU oracle for the fused decode block (test infrastructure, not a product path).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the HIP library and never imports it.
"""
