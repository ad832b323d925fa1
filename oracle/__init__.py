"""CPU oracle for the OD-SGD update path. Test infrastructure only: nothing in
the product package may import this."""
