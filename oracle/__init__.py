"""CPU oracle for the LagKV compression pass.  Test infrastructure only: the
product path (the HIP library and its Python binding) never imports this."""
