"""USP (Ulysses x Ring) attention hot path for MI355X: Python binding over the C-ABI library."""
