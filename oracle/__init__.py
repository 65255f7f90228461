"""CPU oracles for the parity tests -- TEST INFRASTRUCTURE, never imported by the product.

gemm_oracle      fp64-accumulating plain GEMM (C, via ctypes)
selector_oracle  plain-Python CART, labelling and ratio metrics
"""
