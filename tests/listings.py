"""Program text of the paper's listings, as fed unchanged to the CPU oracle and to the library.

The listings themselves (Fig. 2a convolution, Fig. 2b matMul, Fig. 2c max pooling) are the paper's;
the symbols C, Kh, Kw, Sh, Sw are bound to integers by the caller.
"""

CONV2D = """
(transpose
 (squeeze
  (compute dotProd
   (cartProd
    (windows (access activations 1) (shape C Kh Kw) (shape 1 Sh Sw))
    (access weights 1)))
  1)
 (list 0 3 1 2))
"""

MATMUL = """
(compute dotProd
 (cartProd (access activations 1)
           (transpose (access weights 1) (list 1 0))))
"""

MAXPOOL = """
(compute reduceMax
 (windows (access activations 2) (shape Kh Kw) (shape Sh Sw)))
"""

# Fig. 2a on an explicitly zero-padded tensor (padding is an extension of the paper)
CONV2D_PADDED = CONV2D.replace("(access activations 1)", "(access (pad (pad activations 2 Ph Ph) 3 Pw Pw) 1)")
