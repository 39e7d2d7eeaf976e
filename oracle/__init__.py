"""MQGrad hot-path oracle: test infrastructure, not product code.

`oracle.ref` wraps the plain single-threaded C++ in `mqgrad_oracle.cpp`;
`oracle.mdp_ref` restates the paper's MDP agent in numpy.  Only tests, the
smoke check and the benchmark's cpu_baseline leg may import this package.
"""
