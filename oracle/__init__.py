"""CPU oracle for the KV transfer path.  Test infrastructure only: nothing in
the product package imports this."""
