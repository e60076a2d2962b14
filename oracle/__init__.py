"""CPU oracle (test infrastructure only).

Only tests, the smoke check and the benchmark's cpu-baseline leg may import this
package.  It shares no code with the GPU library and never imports it.
"""
