"""MI355X-native Bayesian-Stackelberg commitment sweep (gfx950 HIP kernels behind a C ABI).

``paper_2605_18856_amd.bsse`` is the thin binding over ``libbsse.so``;
``paper_2605_18856_amd.workloads`` draws the seeded synthetic games.  Importing the
package loads no native code; the binding loads the library on first use and raises if
it has not been built.
"""
