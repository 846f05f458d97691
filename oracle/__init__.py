"""CPU oracle for the XConv weight-gradient path.  Test infrastructure only:
the product package never imports this."""
