"""CPU oracle for the decode-step attention path (test infrastructure only).

Only tests, the smoke check and the bench's cpu_baseline leg may import this
package; the product path never does.
"""
