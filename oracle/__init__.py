"""CPU oracle: test infrastructure only.

Only tests/, the smoke check and the bench's cpu_baseline leg may import this
package.  It shares no code with the GPU library and imports nothing from it.
"""
