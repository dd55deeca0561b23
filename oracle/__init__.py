"""CPU checkers (test infrastructure): only the tests, the smoke check and the benchmark's CPU-baseline leg may
import anything from here; the library and its binding never do.

zg_oracle      plain C + ctypes: the mini-batch construction path (sampling, relabel, block CSR, gather, mean)
zg_size_model  numpy/scipy: the graph-aware size model used to provision envelopes
"""
