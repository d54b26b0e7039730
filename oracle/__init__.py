"""CPU fp64 oracle for the BPPSA hot path.  TEST INFRASTRUCTURE ONLY.

Everything in this package is a plain, slow, double-precision statement of what
the HIP library must compute: sequential back-propagation (Section 2.1, Eq. 2
and Eq. 3 of the paper), the exclusive scan it is equivalent to (Section 3.1,
Eq. 4 and Eq. 5), the tree scan of Algorithm 1 written as a recursion as a
second opinion, the sparse transposed Jacobians of Appendix D obtained by
brute force, and one whole training iteration of Section 4.1's RNN.

It shares no code with the HIP path and must never be imported by the product
package: only the tests, the smoke check and the benchmark's cpu_baseline leg
use it.

Pin status (what fixes each function to something other than itself) is listed
in the header of each module.  Functions with no external pin say
"parity unpinned".
"""
