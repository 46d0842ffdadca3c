"""CPU fp64 oracle (test infrastructure only; the product path never imports this).

`oracle.c_oracle`  : plain C loops (oracle/slora_oracle.c) behind ctypes; the timed one.
`oracle.np_oracle` : an independent numpy formulation used to cross-check the C one.
"""
