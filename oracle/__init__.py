"""CPU fp64 oracle for sigmoid / softmax attention.  Test infrastructure only: the product
path never imports this package."""
