"""Block-circulant layers (CirCNN, arXiv 1708.08917) on MI355X: HIP library + ctypes binding."""
