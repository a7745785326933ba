"""CPU oracle for the CurDKV selection path.  Test infrastructure only: the
product (the HIP library and its binding) never imports this package."""
