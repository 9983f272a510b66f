"""CPU oracle (test infrastructure only): plain C reference of the sparse-format
engine plus its ctypes wrapper.  Nothing under the product package imports this."""
