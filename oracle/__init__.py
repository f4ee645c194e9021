"""CPU oracle for the FREE parallel-verification pass.

TEST INFRASTRUCTURE ONLY.  Nothing in the product package may import this
package; only the tests, the smoke check and the cpu-baseline leg of the
benchmark call it.  It shares no code with the HIP path.
"""
