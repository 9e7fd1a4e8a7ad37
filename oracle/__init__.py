"""TEST ORACLE package -- slow, plain CPU reference (float64 cyclic Jacobi) and
the acceptance metrics.  Test infrastructure only: nothing in the product
package imports it."""
